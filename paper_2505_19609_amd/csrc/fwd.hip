// Forward kernel: packed varlen causal attention for one micro-batch
// (local sequences whole, distributed ones as a contiguous query shard against
// the gathered KV prefix -- paper Sec. 4.1).  This is the O(n^2) term of the
// paper's cost model (App. B.2), the thing its scheduler balances.
//
// One workgroup = one work item (a block of BM query rows of one sequence) x
// one query head.  It has 4 wavefronts, each owning 32 query rows, so it covers
// 128 rows at a time; a 256-row item is two such passes, a 64-row item leaves
// two wavefronts to help with staging only.  The key / value prefix is
// streamed in tiles of 64 rows through LDS.
//
// Orientation (see mfma.h): every tile is computed TRANSPOSED so that the
// query index is the MFMA column and therefore lane-local:
//     S^T[j, i] = sum_t K[j,t] Q[i,t]          A = K tile (LDS), B = Q (registers)
//     O^T[t, i] += sum_j V^T[t,j] P^T[j,i]     A = V^T tile (LDS), B = P^T (registers)
// A lane holds one query's 16 scores per 32x32 tile, so the running max, the
// running sum and the rescale of O are plain per-lane scalars, and the S^T
// accumulator registers, once converted to bf16, ARE the B operand of the
// second product (the contraction index j just has to be enumerated the same
// way on the A side, which the V^T LDS layout takes care of).
#include "common.h"
#include "mfma.h"
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
    float scale_log2;  // softmax_scale * log2(e)
};

constexpr int NW = 4;          // wavefronts per workgroup
constexpr int SUB = 32 * NW;   // query rows per pass

template <int D>
__global__ __launch_bounds__(64 * NW, 2) void fwd_kernel(const FwdParams prm)
{
    constexpr int NT = 64 * NW;  // threads
    constexpr int KS = D / 16;   // MFMA k-steps of Q.K^T
    constexpr int TT = D / 32;   // 32-row tiles of O^T
    static_assert(KT == TILE_ROWS, "staging helpers assume 64-row tiles");

    constexpr int TILE_BYTES = TileGeom<D>::BYTES;
    // Two tile buffers, each its own LDS object, and a tile loop unrolled by two
    // so that every access names its buffer statically: the compiler can then
    // tell that the operand reads of one buffer never touch the buffer an
    // asynchronous load is filling, and does not wait for that load first.
    __shared__ __align__(16) unsigned char lds_k0[TILE_BYTES], lds_k1[TILE_BYTES];
    __shared__ __align__(16) unsigned char lds_v0[TILE_BYTES], lds_v1[TILE_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, lives in an SGPR
    const int n = lane & 31, h = lane >> 5;

    // blockIdx -> (item, head).  Consecutive blocks go to consecutive XCDs; the
    // heads of one KV group are Hkv blocks apart so that they share an XCD (and
    // its L2 copy of the K/V tiles) whenever Hkv divides 8 or is a multiple of it.
    const int item_id = blockIdx.x / prm.Hq, hl = blockIdx.x % prm.Hq;
    const int g = prm.Hq / prm.Hkv;
    const int c = hl % prm.Hkv;
    const int head = c * g + hl / prm.Hkv;

    FragAddr<D> fa;
    fa.init(lane);
    TileLoader<D, NT> ld;
    ld.init(tid, (uint32_t)prm.Hkv * D * 2);

    const int4 it = prm.items[item_id];
    const int seq = it.x;
    const int qb = prm.q_begin[seq], ql = prm.q_len[seq], kvl = prm.kv_len[seq];
    const int kbase = prm.cu_k[seq];
    const int item_rows = min(prm.BM, ql - it.y * prm.BM);

    for (int sub = 0; sub * SUB < item_rows; ++sub) {
    const int row0 = it.y * prm.BM + sub * SUB;
    const int qrow0 = it.z + sub * SUB;
    const int rows = min(SUB, ql - row0);
    const int p0 = qb + row0;  // global position of the pass's first query
    const int n_tiles = (p0 + rows + KT - 1) / KT;

    const int wrow0 = 32 * wave;
    const bool wave_active = wrow0 < rows;
    const int my_i = wrow0 + n;
    const int my_pos = p0 + my_i;
    const int w_pmin = p0 + wrow0;
    const int w_pmax = p0 + min(wrow0 + 31, rows - 1);

    // Q fragments (B operand of S^T): this lane's query row, 8 head-dims per k-step.
    bf16x8 qf[KS];
    {
        const uint16_t *qp =
            prm.q + ((size_t)(qrow0 + min(my_i, rows - 1)) * prm.Hq + head) * D + 8 * h;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = as_bf16x8(*(const uint4 *)(qp + 16 * ks));
    }

    const __amdgpu_buffer_rsrc_t rk = ld.rsrc(prm.k + ((size_t)kbase * prm.Hkv + c) * D, kvl);
    const __amdgpu_buffer_rsrc_t rv = ld.rsrc(prm.v + ((size_t)kbase * prm.Hkv + c) * D, kvl);

    f32x16 oacc[TT];
    zero_acc(oacc);
    float m_run = -INFINITY, l_run = 0.0f;
    const float cs = prm.scale_log2;

    // one key tile: start the fetch of the next one into the other buffer, then
    // S^T, online softmax and O^T on the current one
    auto do_tile = [&](int tile, const unsigned char *tk, const unsigned char *tv,
                       unsigned char *nk, unsigned char *nv) __attribute__((always_inline)) {
        const int kv0 = tile * KT;
        if (tile + 1 < n_tiles) {  // lands during the math below
            ld.load(rk, nk, kv0 + KT, tid);
            ld.load(rv, nv, kv0 + KT, tid);
        }

        if (wave_active && kv0 <= w_pmax) {
            f32x16 s[2];
            zero_acc(s);
            // operand fragments are read from LDS in groups ahead of the MFMAs that use them
#pragma unroll
            for (int kh = 0; kh < 2; ++kh) {
                bf16x8 f0[KS / 2], f1[KS / 2];
#pragma unroll
                for (int x = 0; x < KS / 2; ++x) {
                    f0[x] = fa.rows(tk, 0, kh * (KS / 2) + x);
                    f1[x] = fa.rows(tk, 1, kh * (KS / 2) + x);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int x = 0; x < KS / 2; ++x) {  // two independent accumulation chains
                    s[0] = mfma32(f0[x], qf[kh * (KS / 2) + x], s[0]);
                    s[1] = mfma32(f1[x], qf[kh * (KS / 2) + x], s[1]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // first transposed V fragments: their latency hides behind the softmax arithmetic
            bf16x8 fv[TT];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) fv[tt] = fa.cols(tv, tt, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (kv0 + KT - 1 > w_pmin) {  // tile touches the diagonal for this wave
#pragma unroll
                for (int jt = 0; jt < 2; ++jt)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        s[jt][v] = (kv0 + 32 * jt + acc_row(v, h) > my_pos) ? -INFINITY : s[jt][v];
            }
            float mx = s[0][0];
#pragma unroll
            for (int jt = 0; jt < 2; ++jt)
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[jt][v]);
            mx = fmaxf(mx, xor32(mx));
            const float m_new = fmaxf(m_run, mx * cs);
            float rs = 0.0f;
#pragma unroll
            for (int jt = 0; jt < 2; ++jt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = fast_exp2(__builtin_fmaf(s[jt][v], cs, -m_new));
                    s[jt][v] = p;
                    rs += p;
                }
            if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {  // rescale only when a max moved
                const float alpha = fast_exp2(m_run - m_new);
                l_run *= alpha;
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[tt][v] *= alpha;
            }
            l_run += rs;
            m_run = m_new;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kbg = 0; kbg < 4; ++kbg) {
                const bf16x8 pb = acc_to_b(s[kbg >> 1], kbg & 1);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) oacc[tt] = mfma32(fv[tt], pb, oacc[tt]);
                if (kbg < 3) {
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) fv[tt] = fa.cols(tv, tt, kbg + 1);
                }
            }
        }
        wait_vmem();      // my share of the next tile has landed
        __syncthreads();  // ... and everyone's; everyone is done reading this tile
    };

    __syncthreads();  // the previous pass is done with both buffers
    ld.load(rk, lds_k0, 0, tid);
    ld.load(rv, lds_v0, 0, tid);
    wait_vmem();
    __syncthreads();
    for (int tile = 0; tile < n_tiles; tile += 2) {
        do_tile(tile, lds_k0, lds_v0, lds_k1, lds_v1);
        if (tile + 1 < n_tiles) do_tile(tile + 1, lds_k1, lds_v1, lds_k0, lds_v0);
    }

    if (wave_active) {
        const float l_tot = l_run + xor32(l_run);
        const float inv = 1.0f / l_tot;
        if (my_i < rows) {
            store_rows_bf16<TT>(prm.o + ((size_t)(qrow0 + my_i) * prm.Hq + head) * D, oacc, inv, h);
            if (h == 0)
                prm.lse[(size_t)head * prm.total_q + qrow0 + my_i] =
                    (m_run + __log2f(l_tot)) * 0.6931471805599453f;
        }
    }
    }  // pass
}

template <int D>
hipError_t launch_one(const FwdParams &prm, int grid, hipStream_t st)
{
    fwd_kernel<D><<<grid, 64 * NW, 0, st>>>(prm);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd(const skrull_attn_plan_t *p, const void *q, const void *k, const void *v,
                      void *o, float *lse, hipStream_t st)
{
    FwdParams prm;
    prm.q = (const uint16_t *)q; prm.k = (const uint16_t *)k; prm.v = (const uint16_t *)v;
    prm.o = (uint16_t *)o; prm.lse = lse;
    prm.items = (const int4 *)p->fwd_items;
    prm.cu_k = p->cu_k; prm.q_begin = p->q_begin; prm.q_len = p->q_len; prm.kv_len = p->kv_len;
    prm.Hq = p->Hq; prm.Hkv = p->Hkv; prm.total_q = p->total_q; prm.BM = p->BM;
    prm.scale_log2 = p->scale * 1.4426950408889634f;
    const int grid = p->n_fwd * p->Hq;
    if (p->d == 128) return launch_one<128>(prm, grid, st);
    if (p->d == 64) return launch_one<64>(prm, grid, st);
    return hipErrorInvalidValue;
}
