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

// Row-major tile, CH = D/8 chunks of 16 bytes per row.
template <int CH>
__device__ __forceinline__ int rm_off(int row, int chunk)
{
    return (row * CH + (chunk ^ (row & 7))) * 16;
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
