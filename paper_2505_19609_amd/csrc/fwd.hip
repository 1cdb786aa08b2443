// Forward kernel: packed varlen causal attention for one micro-batch
// (local sequences whole, distributed ones as this rank's query segments against
// the gathered KV prefix -- paper Sec. 4.1).  This is the O(n^2) term of the
// paper's cost model (App. B.2), the thing its scheduler balances.
//
// One workgroup = one work item (a block of BM query rows of one sequence) x
// one query head, or a 128-row part of it.  In its large shape it has 8 wavefronts
// (two per SIMD), each owning 32 query rows, so it covers 256 rows; the key / value
// prefix is streamed in tiles of 64 rows through two rings of four LDS slots: two
// tiles are read while the next two are fetched, and the workgroup meets at a
// barrier every second tile.  The small shape (4 wavefronts, two-slot rings, two
// workgroups per compute unit) is described at NW_SMALL below.
//
// Orientation (see mfma.h): every tile is computed TRANSPOSED so that the
// query index is the MFMA column and therefore lane-local:
//     S^T[j, i] = sum_t K[j,t] Q[i,t]          A = K tile (LDS), B = Q (registers)
//     O^T[t, i] += sum_j V^T[t,j] P^T[j,i]     A = V^T tile (LDS), B = P^T (registers)
// A lane holds one query's 16 scores per 32x32 block, so the running max, the
// running sum and the rescale of O are plain per-lane scalars, and the S^T
// accumulator registers, once converted to bf16, ARE the B operand of the
// second product.
//
// Software pipeline.  The unit is a half tile (32 keys).  Step j of a wave
// issues, interleaved in one instruction stream,
//     the 8 MFMAs of S^T(j+1), the 8 MFMAs of O^T += V^T(j-1) P^T(j-1),
//     and the softmax arithmetic of half tile j,
// so that the matrix pipe always has independent work while the vector ALU
// does the exponentials, and LDS operand reads run three MFMA pairs ahead of
// their use.  Steps that touch the start, the end or the causal diagonal of a
// wave's key range take a plain, unpipelined path.
#include <type_traits>

#include "common.h"
#include "mfma.h"
#include "queue.h"
#include "tiles.h"

namespace {

constexpr int KT = 64;  // key rows per tile

struct FwdParams {
    const uint16_t *q, *k, *v;
    uint16_t *o;
    float *lse;
    const int4 *items;
    const int32_t *cu_k, *q_begin, *q_len, *kv_len;
    int32_t Hq, Hkv, total_q, BM;
    int32_t variant;  // 0: 4 wavefronts, 128 rows per workgroup; 1: 8 wavefronts, 256 rows
    float scale_log2;  // softmax_scale * log2(e)
    WgTrace *trace;    // null, or one record per work item (measurement aid)
    WorkQueue *queue;  // work queue of the persistent launch, zeroed before use
    int32_t n_work;    // work items: what a plain grid would have as workgroups
};

// Two shapes of the one kernel.  Large: 8 wavefronts = 256 query rows per workgroup and
// 4 ring slots per operand (two tiles being read, two being fetched; a barrier every
// second tile); its 139 KB of LDS leave room for one workgroup per compute unit.  Small:
// 4 wavefronts = 128 rows (a larger item is split over two workgroups) and 2 ring slots
// (fetch one tile ahead, a barrier every tile), 70 KB, so that two workgroups share a
// compute unit and the start-up, drain and barrier waits of one (most of the run time of
// a short sequence) hide behind the other.  The plan chooses per micro-batch.
constexpr int NW_LARGE = 8, NSLOT_LARGE = 4;
constexpr int NW_SMALL = 4, NSLOT_SMALL = 2;

// max / sum of a value over the two halves of the wavefront (lanes l and l ^ 32)
// without going through LDS: two copies of x, the upper half of the first
// swapped with the lower half of the second, then the two combined.  Written out
// whole, with the two idle cycles the swap needs after a vector write of its
// operands: the compiler's builtin for the swap hands back its first result for
// both when given one value twice.
__device__ __forceinline__ float max_halves(float x)
{
    float r, t;
    asm volatile("v_mov_b32 %0, %2\n\tv_mov_b32 %1, %2\n\ts_nop 1\n\t"
                 "v_permlane32_swap_b32 %0, %1\n\tv_max_f32 %0, %0, %1"
                 : "=&v"(r), "=&v"(t) : "v"(x));
    return r;
}
__device__ __forceinline__ float sum_halves(float x)
{
    float r, t;
    asm volatile("v_mov_b32 %0, %2\n\tv_mov_b32 %1, %2\n\ts_nop 1\n\t"
                 "v_permlane32_swap_b32 %0, %1\n\tv_add_f32 %0, %0, %1"
                 : "=&v"(r), "=&v"(t) : "v"(x));
    return r;
}

// Two scores -> two probabilities (exp2 of score * c - m), in two parts so that
// each part can sit behind one MFMA of a pipelined step: part one is the two
// multiply-adds and exponentials, part two adds the results to rs and packs
// them to bf16.  Written out so that the instructions stay where the kernel puts
// them (plain arithmetic would be moved to its first use, i.e. behind all the
// MFMAs of the step).  Each exponential has an instruction between it and the
// first use of its result, which is what this target asks for after a
// transcendental.
__device__ __forceinline__ void softmax_exp2(float s0, float s1, float c, float m, float &t0, float &t1)
{
    asm volatile("v_fma_f32 %0, %2, %4, -%5\n\t"
                 "v_fma_f32 %1, %3, %4, -%5\n\t"
                 "v_exp_f32 %0, %0\n\t"
                 "v_exp_f32 %1, %1"
                 : "=&v"(t0), "=&v"(t1)
                 : "v"(s0), "v"(s1), "s"(c), "v"(m));
}
__device__ __forceinline__ uint32_t softmax_sum_pack(float t0, float t1, float &ra, float &rb)
{
    uint32_t pk;
    asm volatile("v_add_f32 %1, %1, %3\n\t"
                 "v_add_f32 %2, %2, %4\n\t"
                 "v_cvt_pk_bf16_f32 %0, %3, %4"
                 : "=v"(pk), "+v"(ra), "+v"(rb)
                 : "v"(t0), "v"(t1));
    return pk;
}

template <int D, int NW, int NSLOT>
__device__ __forceinline__ void fwd_work(const FwdParams &prm, const int bid)
{
    static_assert(NSLOT == 2 || NSLOT == 4, "ring logic below covers two and four slots");
    constexpr int SM = NSLOT - 1;  // slot of tile t: t & SM
    constexpr int KS = D / 16;   // MFMA k-steps of Q.K^T
    constexpr int TT = D / 32;   // 32-row tiles of O^T
    static_assert(KT == TILE_ROWS, "staging helpers assume 64-row tiles");
    static_assert(KS == 2 * TT, "a step pairs one S MFMA with one O MFMA");
    typedef TileGeom<D> G;
    constexpr int TB = G::BYTES;
    constexpr int HALF = 32 * G::ROWB;  // byte offset of a tile's second 32 rows
    typedef RingLoader<D, NW> Loader;

    __shared__ __align__(16) unsigned char lds_k[NSLOT][TB];
    __shared__ __align__(16) unsigned char lds_v[NSLOT][TB];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, lives in an SGPR
    const int n = lane & 31, h = lane >> 5;

    // work index -> (item, head).  Consecutive blocks go to consecutive XCDs; the
    // heads of one KV group are Hkv blocks apart so that they share an XCD (and
    // its L2 copy of the K/V tiles) whenever Hkv divides 8 or is a multiple of it.
    // an item of more rows than the workgroup covers is split over `subs` workgroups
    const int subs = (prm.BM + 32 * NW - 1) / (32 * NW);
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

    const int4 it = prm.items[item_id];
    const int seq = it.x;
    const int qb = prm.q_begin[seq], ql = prm.q_len[seq], kvl = prm.kv_len[seq];
    const int kbase = prm.cu_k[seq];
    const int item_rows = min(prm.BM, ql - it.y * prm.BM);
    const float cs = prm.scale_log2;

    const int row0 = it.y * prm.BM + sub * 32 * NW;
    const int qrow0 = it.z + sub * 32 * NW;
    const int rows = min(32 * NW, item_rows - sub * 32 * NW);
    if (rows <= 0) return;  // the item ends before this part (the whole workgroup leaves)
    const uint64_t trace_t0 = trace_begin(prm.trace);
    const int p0 = qb + row0;  // global position of the pass's first query
    const int n_tiles = (p0 + rows + KT - 1) / KT;

    const int wrow0 = 32 * wave;
    const bool wave_active = wrow0 < rows;
    const int my_i = wrow0 + n;
    const int w_pmin = p0 + wrow0;
    const int w_pmax = p0 + min(wrow0 + 31, rows - 1);
    // half tiles (32 keys) of this wave: 0..L hold a visible key, those below n_full only visible keys
    const int L = wave_active ? w_pmax / 32 : -1;
    const int n_full = wave_active ? (w_pmin + 1) / 32 : 0;

    // Q fragments (B operand of S^T): this lane's query row, 8 head-dims per k-step
    // (loaded below, behind the first tile fetches)
    bf16x8 qf[KS];
    const i32x4 rk = ld.rsrc(prm.k + ((size_t)kbase * prm.Hkv + c) * D, kvl);
    const i32x4 rv = ld.rsrc(prm.v + ((size_t)kbase * prm.Hkv + c) * D, kvl);

    f32x16 oacc[TT];
    zero_acc(oacc);
    float m_run = -INFINITY, l_run = 0.0f;

    // ---- softmax pieces ---------------------------------------------------
    auto row_max = [&](const f32x16 &s) __attribute__((always_inline)) {
        float mx = fmaxf(s[0], s[1]);
#pragma unroll
        for (int v = 2; v < 16; v += 2) mx = __builtin_fmaxf(__builtin_fmaxf(mx, s[v]), s[v + 1]);
        mx = max_halves(mx) * cs;
        // The running maximum only has to bound the scores loosely: it moves when a
        // score exceeds it by more than 2^8 (exponentials then stay below 256, far
        // inside fp32 and bf16 range), so after the first tiles O is hardly ever rescaled.
        return mx > m_run + 8.0f ? mx : m_run;
    };
    // rescale of the running sum and of O when some lane's maximum moved
    auto finish = [&](float m_new, float rs) __attribute__((always_inline)) {
        if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {
            const float alpha = fast_exp2(m_run - m_new);
            l_run *= alpha;
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[tt][v] *= alpha;
        }
        l_run += rs;
        m_run = m_new;
    };

    // ---- pipelined step j: S(j+1) from kp, softmax(j) on s_in, O += V(j-1) P(j-1) from vp
    // FIRST: first step of a period (reads its first operands itself and, at the
    // end, those of the second step from kp2 / vp2); otherwise they are in kf / vf.
    auto steady = [&](auto first_tag, const unsigned char *kp, const unsigned char *vp,
                      const unsigned char *kp2, const unsigned char *vp2, const f32x16 &s_in,
                      f32x16 &s_out, const bf16x8 (&p_in)[2], bf16x8 (&p_out)[2], bf16x8 (&kf)[4],
                      bf16x8 (&vf)[4]) __attribute__((always_inline)) {
        constexpr bool FIRST = decltype(first_tag)::value;
        if (FIRST) {
#pragma unroll
            for (int x = 0; x < 3; ++x) {
                kf[x] = fa.rows(kp, 0, x);
                vf[x] = fa.cols(vp, x % TT, x / TT);
            }
        }
        SB();
        float rs0 = 0.0f, rs1 = 0.0f;
        uint32_t pw[8];
        SB();
#pragma unroll
        for (int i = 0; i < KS; ++i) {
            // one MFMA, a few vector instructions, one MFMA, a few more: the vector
            // work of this step's share of the 16 scores runs behind the matrix pipe
            constexpr int EPS = 16 / KS;  // scores per step (2 or 4)
            float t[EPS];
            if (i == 0) {
                f32x16 z;
#pragma unroll
                for (int v = 0; v < 16; ++v) z[v] = 0.0f;
                s_out = mfma32(kf[0], qf[0], z);
            } else {
                s_out = mfma32(kf[i % 4], qf[i], s_out);
            }
#pragma unroll
            for (int e = 0; e < EPS; e += 2)
                softmax_exp2(s_in[EPS * i + e], s_in[EPS * i + e + 1], cs, m_run, t[e], t[e + 1]);
            SB();
            oacc[i % TT] = mfma32(vf[i % 4], p_in[i / TT], oacc[i % TT]);
#pragma unroll
            for (int e = 0; e < EPS; e += 2) pw[(EPS * i + e) >> 1] = softmax_sum_pack(t[e], t[e + 1], rs0, rs1);
            const int nx = i + 3;
            if (nx < KS) {
                kf[nx % 4] = fa.rows(kp, 0, nx);
                vf[nx % 4] = fa.cols(vp, nx % TT, nx / TT);
            } else if (FIRST) {
                kf[nx % 4] = fa.rows(kp2, 0, nx - KS);
                vf[nx % 4] = fa.cols(vp2, (nx - KS) % TT, (nx - KS) / TT);
            }
            SB();
        }
        float rs = rs0 + rs1;
        // The step took its exponentials against the bound of the steps before it, without
        // looking for the maximum of its scores first (that chain of maxima was a seventh of the
        // step's vector instructions).  The bound only has to hold loosely, and the sum the step
        // forms anyway tells when it no longer does: a row whose probabilities of this step add up
        // to more than 2^10 in either half of the wavefront (or overflowed) takes its true
        // maximum as the new bound, and the step's probabilities are formed again from the
        // scores, which are still in their registers.  After the first tiles this hardly ever
        // happens; rows that keep their bound form the same values again.
        constexpr float kSumBound = 1024.0f;
        float m_new = m_run;
        if (__builtin_amdgcn_ballot_w64(!(rs <= kSumBound)) != 0) {
            float mx = fmaxf(s_in[0], s_in[1]);
#pragma unroll
            for (int v = 2; v < 16; v += 2) mx = __builtin_fmaxf(__builtin_fmaxf(mx, s_in[v]), s_in[v + 1]);
            mx = max_halves(mx) * cs;
            const bool moved = !(max_halves(rs) <= kSumBound);
            m_new = moved ? fmaxf(mx, m_run) : m_run;
            rs0 = 0.0f;
            rs1 = 0.0f;
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
                float t0, t1;
                softmax_exp2(s_in[v], s_in[v + 1], cs, m_new, t0, t1);
                pw[v >> 1] = softmax_sum_pack(t0, t1, rs0, rs1);
            }
            rs = rs0 + rs1;
        }
        finish(m_new, rs);
        p_out[0] = as_bf16x8(make_uint4(pw[0], pw[1], pw[2], pw[3]));
        p_out[1] = as_bf16x8(make_uint4(pw[4], pw[5], pw[6], pw[7]));
    };

    // ---- plain step j with run-time guards (start, end and diagonal of the wave's range)
    auto generic = [&](int j, const unsigned char *kp, const unsigned char *vp, const f32x16 &s_in,
                       f32x16 &s_out, const bf16x8 (&p_in)[2], bf16x8 (&p_out)[2]) __attribute__((always_inline)) {
        if (j - 1 >= 0 && j - 1 <= L) {  // O += V(j-1) P(j-1)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) oacc[tt] = mfma32(fa.cols(vp, tt, kb), p_in[kb], oacc[tt]);
                SB();
            }
        }
        if (j + 1 <= L) {  // S(j+1)
#pragma unroll
            for (int v = 0; v < 16; ++v) s_out[v] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s_out = mfma32(fa.rows(kp, 0, ks), qf[ks], s_out);
                if (ks % 4 == 3) SB();
            }
        }
        if (j >= 0 && j <= L) {  // softmax(j)
            f32x16 s = s_in;
            if (j >= n_full) {  // half tile touches the diagonal for this wave
                // relative position from an opaque copy of the lane index: the sixteen
                // per-register thresholds are formed here rather than kept for the whole kernel
                int li = lane;
                asm volatile("" : "+v"(li));
                const int rel = p0 + wrow0 + (li & 31) - 32 * j - 4 * (li >> 5);  // this lane's query position - 32j - 4h
#pragma unroll
                for (int v = 0; v < 16; ++v) s[v] = (8 * (v >> 2) + (v & 3) > rel) ? -INFINITY : s[v];
            }
            const float m_new = row_max(s);
            float rs = 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                s[v] = fast_exp2(__builtin_fmaf(s[v], cs, -m_new));
                rs += s[v];
            }
            p_out[0] = acc_to_b(s, 0);
            p_out[1] = acc_to_b(s, 1);
            finish(m_new, rs);
        }
    };

    // Four slots: the fetch group issued at the start of an even period t is K tiles t+2,
    // t+3 and V tiles t+1, t+2 (tiles past the end read as zero), into the slots that the
    // two periods before the last barrier have left.  Two slots: every period t starts by
    // fetching K tile t+1 and V tile t into the slots period t-1 has left.
    auto fetch = [&](int t) __attribute__((always_inline)) {
        if (NSLOT == 4) {
            ld.load(rk, ring_k + (uint32_t)((t + 2) & 3) * TB, (t + 2) * KT, wave);
            ld.load(rv, ring_v + (uint32_t)((t + 1) & 3) * TB, (t + 1) * KT, wave);
            ld.load(rk, ring_k + (uint32_t)((t + 3) & 3) * TB, (t + 3) * KT, wave);
            ld.load(rv, ring_v + (uint32_t)((t + 2) & 3) * TB, (t + 2) * KT, wave);
        } else {
            ld.load(rk, ring_k + (uint32_t)((t + 1) & 1) * TB, (t + 1) * KT, wave);
            ld.load(rv, ring_v + (uint32_t)(t & 1) * TB, t * KT, wave);
        }
    };

    // Start-up: the tiles of the first period.  The rest of period 0's fetch group follows after
    // the barrier below, because until then its slots stage this item's rows of Q.
    ld.load(rk, ring_k, 0, wave);  // K tile 0
    if (NSLOT == 4) ld.load(rk, ring_k + TB, KT, wave);  // K tile 1
    ld.load(rv, ring_v, 0, wave);  // V tile 0
    // this wave's staging region: half a ring slot that holds no tile yet (four slots: K slots
    // 2-3 for waves 0-3, V slots 1-2 for waves 4-7; two slots: K slot 1 for waves 0-1, V slot 1
    // for waves 2-3)
    typedef WaveStage<D> Stage;
    static_assert(2 * Stage::BYTES == TB, "two staging regions per ring slot");
    static_assert((NSLOT == 4 && NW == 8) || (NSLOT == 2 && NW == 4), "staging regions are laid out for these shapes");
    const uint32_t stage = NSLOT == 4 ? (wave < 4 ? ring_k + 2 * TB + (uint32_t)wave * Stage::BYTES
                                                  : ring_v + TB + (uint32_t)(wave - 4) * Stage::BYTES)
                                      : (wave < 2 ? ring_k + TB + (uint32_t)wave * Stage::BYTES
                                                  : ring_v + TB + (uint32_t)(wave - 2) * Stage::BYTES);
    {
        Stage st;
        st.init(lane);
        u32x4 vq[Stage::N];
        st.load(vq, prm.q + ((size_t)qrow0 * prm.Hq + head) * D, (uint32_t)prm.Hq * D * 2, wrow0, rows);
        st.put(stage, vq);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = fa.rows_at(stage, ks);
    }
    // Everything issued so far has to land here: the compiler's own count of
    // outstanding loads must be zero before the loops, or the waits it places
    // for these fragments would also wait for the tile fetches in flight.
    wait_vmem();
    __syncthreads();
    // the staging regions are free again: what is left of period 0's fetch group
    if (NSLOT == 4) {
        if (1 < n_tiles) fetch(0);
    } else {
        ld.load(rk, ring_k + TB, KT, wave);  // K tile 1
    }

    f32x16 sx, sy;         // S of the current / next half tile, ping-pong
    bf16x8 px[2], py[2];   // P of the previous / current half tile, ping-pong
#pragma unroll
    for (int v = 0; v < 16; ++v) { sx[v] = 0.0f; sy[v] = 0.0f; }
    {
        const uint4 z4 = make_uint4(0, 0, 0, 0);
        px[0] = px[1] = py[0] = py[1] = as_bf16x8(z4);
    }

    // Period t: steps 2t-1 and 2t, i.e. S of both halves of K tile t and the
    // O update with both halves of V tile t-1.  K tile t sits in slot t % NSLOT,
    // V tile t-1 in slot (t-1) % NSLOT.  With four slots fetches are issued, and the
    // workgroup meets at a barrier, every second period: an even period starts by fetching
    // the tiles of the next two periods into the slots the previous two have left, an odd
    // period ends with the wait for them and the barrier.  With two slots every period
    // fetches for the next one and ends with the wait and the barrier.
    auto period_begin = [&](int t) __attribute__((always_inline)) {
        if (t == 0) return;  // issued at start-up
        if (NSLOT == 4) {
            if ((t & 1) == 0 && t + 1 < n_tiles) fetch(t);  // V tile t+1 exists
        } else {
            if (t < n_tiles) fetch(t);  // V tile t exists
        }
    };
    auto period_end = [&](int t) __attribute__((always_inline)) {
        if (NSLOT == 2 || (t & 1)) {
            wait_vmem();      // my share of the tiles of the next period(s) has landed
            __syncthreads();  // ... and everyone's; everyone is done with the tiles they replace
        }
    };
    // periods whose two steps are fully inside the wave's unmasked range
    const int t_steady_end = min((L - 1) / 2, (n_full - 1) / 2);  // last t with 2t+1 <= L and 2t < n_full
    // one copy of the plain step, run for both halves of a period; its results
    // are moved back so that a period always starts from sx / px
    auto plain_period = [&](int t) __attribute__((always_inline)) {
        period_begin(t);
        const unsigned char *tk = lds_k[t & SM], *tv = lds_v[(t - 1) & SM];
#pragma unroll 1
        for (int hh = 0; hh < 2; ++hh) {
            generic(2 * t - 1 + hh, tk + hh * HALF, tv + hh * HALF, sx, sy, px, py);
            sx = sy;
            px[0] = py[0];
            px[1] = py[1];
        }
        period_end(t);
    };
    plain_period(0);
    int t = 1;
    // the pipelined loop proper: S and P ping-pong between two register sets
    for (; t <= t_steady_end; ++t) {
        period_begin(t);
        const unsigned char *tk = lds_k[t & SM], *tv = lds_v[(t - 1) & SM];
        bf16x8 kf[4], vf[4];  // operand fragments in flight
        steady(std::true_type{}, tk, tv, tk + HALF, tv + HALF, sx, sy, px, py, kf, vf);
        steady(std::false_type{}, tk + HALF, tv + HALF, tk, tv, sy, sx, py, px, kf, vf);
        period_end(t);
    }
#pragma unroll 1
    for (; t <= n_tiles; ++t) plain_period(t);

    __syncthreads();  // nobody reads a tile any more: the staging regions are free
    if (wave_active) {
        const float l_tot = sum_halves(l_run);
        const float inv = 1.0f / l_tot;
        // the output addresses are formed here, after the loop, from opaque copies,
        // so that nothing of them occupies registers during the loop
        int li = lane;
        asm volatile("" : "+v"(li));
        const int on = li & 31, oh = li >> 5, oi = wrow0 + on;
        Stage st;
        st.init(li);
        st.put_acc(stage, oacc, inv, on, oh);
        st.store(stage, prm.o + ((size_t)qrow0 * prm.Hq + head) * D, (uint32_t)prm.Hq * D * 2, wrow0, rows);
        if (oh == 0 && oi < rows)
            prm.lse[(size_t)head * prm.total_q + qrow0 + oi] = (m_run + __log2f(l_tot)) * 0.6931471805599453f;
    }
    trace_end(prm.trace, trace_t0, bid);
}

template <int D, int NW, int NSLOT>
__global__ __launch_bounds__(64 * NW, 2) void fwd_kernel(const FwdParams prm)
{
    __shared__ int work_slot;
    work_loop(prm.queue, prm.n_work, &work_slot,
              [&](int w) __attribute__((always_inline)) { fwd_work<D, NW, NSLOT>(prm, w); });
}

template <auto Kernel>
hipError_t launch_shape(FwdParams prm, int threads, hipStream_t st)
{
    const bool queued = wants_queue<Kernel>(threads, prm.n_work);
    if (queued) {
        queue_reset_kernel<<<1, 64, 0, st>>>(prm.queue, 1);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    } else {
        prm.queue = nullptr;
    }
    return launch_work<Kernel>(threads, prm.n_work, queued, prm, st);
}

template <int D>
hipError_t launch_one(const FwdParams &prm, hipStream_t st)
{
    if (prm.variant == 0) return launch_shape<fwd_kernel<D, NW_SMALL, NSLOT_SMALL>>(prm, 64 * NW_SMALL, st);
    return launch_shape<fwd_kernel<D, NW_LARGE, NSLOT_LARGE>>(prm, 64 * NW_LARGE, st);
}

}  // namespace

int grid_fwd(const skrull_attn_plan_t *p)
{
    const int subs = p->wg_query_rows == 32 * NW_SMALL ? (p->BM + 32 * NW_SMALL - 1) / (32 * NW_SMALL) : 1;
    return p->n_fwd * p->Hq * subs;
}

hipError_t launch_fwd(const skrull_attn_plan_t *p, const void *q, const void *k, const void *v,
                      void *o, float *lse, hipStream_t st, WgTrace *trace)
{
    FwdParams prm;
    prm.q = (const uint16_t *)q; prm.k = (const uint16_t *)k; prm.v = (const uint16_t *)v;
    prm.o = (uint16_t *)o; prm.lse = lse;
    prm.items = (const int4 *)p->fwd_items;
    prm.cu_k = p->cu_k; prm.q_begin = p->q_begin; prm.q_len = p->q_len; prm.kv_len = p->kv_len;
    prm.Hq = p->Hq; prm.Hkv = p->Hkv; prm.total_q = p->total_q; prm.BM = p->BM;
    prm.scale_log2 = p->scale * 1.4426950408889634f;
    prm.trace = trace;
    prm.variant = p->wg_query_rows == 32 * NW_SMALL ? 0 : 1;
    prm.n_work = grid_fwd(p);
    // One of the plan's queue slots per call, taken in turn, so that forward calls of one plan
    // that overlap on different streams do not share a queue.
    prm.queue = p->fwd_queues + (__atomic_fetch_add(&const_cast<skrull_attn_plan_t *>(p)->fwd_calls, 1u, __ATOMIC_RELAXED) % SKRULL_FWD_QUEUE_SLOTS);
    if (p->d == 128) return launch_one<128>(prm, st);
    if (p->d == 64) return launch_one<64>(prm, st);
    return hipErrorInvalidValue;
}
