// LDS tile staging shared by the attention kernels.
//
// A tile is 64 rows (keys, or queries in the dK/dV kernel) x D bf16.  It is
// fetched from global memory as "quad units": one thread takes 4 consecutive
// rows x 8 consecutive columns (four 16-byte loads).  From those registers it
// can write
//   * the row-major copy  (A operand of products that contract over D), and/or
//   * the transposed copy (A operand of products that contract over the 64
//     rows), four rows packed per 8-byte store.
// Both copies are XOR-swizzled at 16-byte granularity so that the MFMA operand
// reads (16 bytes per lane) and the staging writes are free of bank conflicts.
#pragma once

#include "mfma.h"

constexpr int TILE_ROWS = 64;

// Row-major tile, CH = D/8 chunks of 16 bytes per row.  LDS has 64 banks of 4
// bytes (a 256-byte line); a wave's 16-byte reads are served 16 lanes at a time
// and its 8-byte reads 32 lanes at a time, so a group is conflict-free when its
// 16-byte slots are distinct modulo 256 bytes.  The chunk index is XOR-ed with
// a function of the row chosen so that
//   * 16 consecutive rows read at the same chunk (MFMA operand reads), and
//   * 4 consecutive rows x 4 consecutive chunks (transposing reads)
// both touch 16 different slots.  At d=128 a row is one line, so the function
// must take 16 values over 16 rows; at d=64 two rows share a line and 8 values
// over 16 rows suffice.
template <int CH>
__device__ __forceinline__ int row_swizzle(int row)
{
    if (CH == 16) return ((row & 3) << 2) | ((row >> 2) & 3);
    return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
}

template <int CH>
__device__ __forceinline__ int rm_off(int row, int chunk)
{
    return (row * CH + (chunk ^ row_swizzle<CH>(row))) * 16;
}

// Transposing fragment read from a ROW-MAJOR tile (ds_read_b64_tr_b16): returns
// the A operand of a product that contracts over the tile's rows.  For the
// 32-column block tt and the 16-row block kbg, lane (n = lane%32, h = lane/32)
// receives column 32*tt+n of rows 16*kbg + {4h..4h+3, 8+4h..8+4h+3}, i.e. the
// rows its accumulator registers 8*(kbg%2)..+7 of a 32x32 result stand for.
// The instruction works on groups of 16 lanes: lane s of a group supplies the
// address of 4 consecutive columns of one row; lane l receives element l%4 of
// the rows supplied by lanes l/4, l/4+4, l/4+8, l/4+12.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

template <int CH>
__device__ __forceinline__ bf16x8 frag_tr_rm(const unsigned char *lds, int tt, int kbg, int lane)
{
    const int grp = lane >> 4, s = lane & 15, h = grp >> 1;
    const int chunk = 4 * tt + 2 * (grp & 1) + ((s & 3) >> 1);
    const int row = 16 * kbg + 4 * h + (s >> 2);
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr_t;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_ptr_t)(lds + rm_off<CH>(row, chunk) + 8 * (s & 1)));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_ptr_t)(lds + rm_off<CH>(row + 8, chunk) + 8 * (s & 1)));
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// Transposed tile: row t = column of the source (0..D-1); 8 chunks = 64 source
// rows in permuted order.  Within each group of 16 source rows the four quads
// are stored in order 0,2,1,3: a lane of half h then finds, in the 16 bytes at
// chunk 2*kb+h, exactly the 8 rows {4h..4h+3, 8+4h..8+4h+3} (+16*kb) that its
// accumulator registers 8*kb..8*kb+7 of a 32x32 MFMA result correspond to.
__device__ __forceinline__ int tr_off(int t, int chunk)
{
    return (t * 8 + (chunk ^ ((t ^ (t >> 3)) & 7))) * 16;
}

// Asynchronous global -> LDS copy of one 64-row x D tile in the row-major
// swizzled layout (global_load_lds_dwordx4: no data registers, no LDS store
// instructions).  One such instruction makes a wave write 64 consecutive
// 16-byte LDS slots, slot = base + lane, from per-lane global addresses; the
// swizzle is therefore applied on the global side: the lane that fills slot P
// fetches the chunk that belongs there.  Rows beyond row_last are clamped (the
// callers mask them).  Completion: s_waitcnt vmcnt(0) then a workgroup barrier.
// `base` must be wave-uniform (row 0 of the sequence, already offset to the head).
template <int D, int NT>
__device__ __forceinline__ void tile_load_async(unsigned char *lds, const uint16_t *base,
                                                uint32_t stride, int row0, int row_last, int tid)
{
    constexpr int CH = D / 8;
    constexpr int PER = TILE_ROWS * CH / NT;
    typedef void __attribute__((address_space(3))) * lds_void_t;
    const int wave_first = tid & ~63;
#pragma unroll
    for (int x = 0; x < PER; ++x) {
        const int P = x * NT + tid;
        const int row = P / CH, chunk = (P % CH) ^ row_swizzle<CH>(row);
        // 32-bit element offset from a wave-uniform base (the plan guarantees that
        // one sequence of one tensor spans fewer than 2^31 elements)
        const uint32_t eoff = (uint32_t)min(row0 + row, row_last) * stride + (uint32_t)(chunk * 8);
        const uint16_t *g = base + eoff;
        __builtin_amdgcn_global_load_lds((const void *)g, (lds_void_t)(lds + (x * NT + wave_first) * 16),
                                         16, 0, 0);
    }
}

// Wait until this wave's outstanding global (and global->LDS) loads have landed.
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

template <int D, int NT>
struct QuadStage {
    static constexpr int CH = D / 8;
    static constexpr int UNITS = (TILE_ROWS / 4) * CH;
    static constexpr int UPT = (UNITS + NT - 1) / NT;
    uint32_t r[UPT][4][4];

    // base: element pointer to column 0 of row 0 of the source (already offset
    // to the head); stride: elements between consecutive rows; rows row0..row0+63
    // are fetched, clamped to row_last (the clamped rows are masked by the caller).
    __device__ __forceinline__ void load(const uint16_t *base, size_t stride, int row0,
                                         int row_last, int tid)
    {
#pragma unroll
        for (int y = 0; y < UPT; ++y) {
            const int u = tid + y * NT;
            if (UNITS % NT == 0 || u < UNITS) {
                const int qd = u / CH, tg = u % CH;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int row = min(row0 + 4 * qd + q, row_last);
                    const uint4 t4 = *(const uint4 *)(base + (size_t)row * stride + tg * 8);
                    r[y][q][0] = t4.x; r[y][q][1] = t4.y; r[y][q][2] = t4.z; r[y][q][3] = t4.w;
                }
            }
        }
    }

    __device__ __forceinline__ void store_rm(unsigned char *lds, int tid) const
    {
#pragma unroll
        for (int y = 0; y < UPT; ++y) {
            const int u = tid + y * NT;
            if (UNITS % NT == 0 || u < UNITS) {
                const int qd = u / CH, tg = u % CH;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *(uint4 *)(lds + rm_off<CH>(4 * qd + q, tg)) =
                        make_uint4(r[y][q][0], r[y][q][1], r[y][q][2], r[y][q][3]);
            }
        }
    }

    __device__ __forceinline__ void store_tr(unsigned char *lds, int tid) const
    {
#pragma unroll
        for (int y = 0; y < UPT; ++y) {
            const int u = tid + y * NT;
            if (UNITS % NT == 0 || u < UNITS) {
                const int qd = u / CH, tg = u % CH;
                const int q4 = qd & 3;
                const int chunk = 2 * (qd >> 2) + (q4 & 1), half = q4 >> 1;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int w = e >> 1;
                    const uint32_t a0 = r[y][0][w], a1 = r[y][1][w], a2 = r[y][2][w], a3 = r[y][3][w];
                    uint2 o2;
                    if (e & 1) {
                        o2.x = (a0 >> 16) | (a1 & 0xffff0000u);
                        o2.y = (a2 >> 16) | (a3 & 0xffff0000u);
                    } else {
                        o2.x = (a0 & 0xffffu) | (a1 << 16);
                        o2.y = (a2 & 0xffffu) | (a3 << 16);
                    }
                    *(uint2 *)(lds + tr_off(8 * tg + e, chunk) + 8 * half) = o2;
                }
            }
        }
    }
};

// Per-lane byte offsets of the MFMA operand fragments inside a row-major tile,
// computed once per kernel.  Everything that varies inside the hot loops (which
// 32-row block, which 16-row block, which of two adjacent tiles) is then a
// compile-time constant added to one of these, i.e. an instruction immediate:
//   operand rows 32*b+n, k-step ks          : rm[ks] + b * 32*ROWB
//   transposed, column block tt, rows 16*kbg : trl[tt] / trh[tt] + kbg * 16*ROWB
// (the swizzle only looks at the row modulo 16, so adding 16 or 32 rows keeps it).
template <int D>
struct FragAddr {
    static constexpr int CH = D / 8, KS = D / 16, TT = D / 32, ROWB = D * 2;
    int rm[KS];
    int trl[TT], trh[TT];

    __device__ __forceinline__ void init(int lane)
    {
        const int n = lane & 31, h = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) rm[ks] = rm_off<CH>(n, 2 * ks + h);
        const int grp = lane >> 4, s = lane & 15;
        const int row = 4 * (grp >> 1) + (s >> 2);
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int chunk = 4 * tt + 2 * (grp & 1) + ((s & 3) >> 1);
            trl[tt] = rm_off<CH>(row, chunk) + 8 * (s & 1);
            trh[tt] = rm_off<CH>(row + 8, chunk) + 8 * (s & 1);
        }
    }
    // rows 32*b + n of the tile at `t`, k-step ks
    __device__ __forceinline__ bf16x8 rows(const unsigned char *t, int b, int ks, int extra = 0) const
    {
        return *(const bf16x8 *)(t + rm[ks] + b * (32 * ROWB) + extra);
    }
    // transposed fragment: column block tt, row block kbg (see frag_tr_rm)
    __device__ __forceinline__ bf16x8 cols(const unsigned char *t, int tt, int kbg, int extra = 0) const
    {
        typedef s16x4 __attribute__((address_space(3))) * lds_ptr_t;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(t + trl[tt] + kbg * (16 * ROWB) + extra));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(t + trh[tt] + kbg * (16 * ROWB) + extra));
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, both);
    }
};

// A-operand fragment reads (16 bytes per lane), n = lane % 32, h = lane / 32.
template <int CH>
__device__ __forceinline__ bf16x8 frag_rm(const unsigned char *lds, int row, int ks, int h)
{
    return *(const bf16x8 *)(lds + rm_off<CH>(row, 2 * ks + h));
}
__device__ __forceinline__ bf16x8 frag_tr(const unsigned char *lds, int t, int kbg, int h)
{
    return *(const bf16x8 *)(lds + tr_off(t, 2 * kbg + h));
}

// Accumulator registers 8*kb .. 8*kb+7 of a 32x32 result -> bf16 B operand.
__device__ __forceinline__ bf16x8 acc_to_b(const f32x16 &s, int kb)
{
    uint4 pk;
    pk.x = pack_bf16(s[8 * kb + 0], s[8 * kb + 1]);
    pk.y = pack_bf16(s[8 * kb + 2], s[8 * kb + 3]);
    pk.z = pack_bf16(s[8 * kb + 4], s[8 * kb + 5]);
    pk.w = pack_bf16(s[8 * kb + 6], s[8 * kb + 7]);
    return as_bf16x8(pk);
}

// Store a 32-column (t) x 32-row accumulator tile set as bf16 rows of a
// [rows, H, D] tensor: this lane's row pointer `dst` (column 0), its half h.
template <int TT>
__device__ __forceinline__ void store_rows_bf16(uint16_t *dst, const f32x16 (&acc)[TT], float mul, int h)
{
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int vb = 0; vb < 4; ++vb) {
            uint2 w;
            w.x = pack_bf16(acc[tt][4 * vb + 0] * mul, acc[tt][4 * vb + 1] * mul);
            w.y = pack_bf16(acc[tt][4 * vb + 2] * mul, acc[tt][4 * vb + 3] * mul);
            *(uint2 *)(dst + 32 * tt + 8 * vb + 4 * h) = w;
        }
}

template <int N>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
}
