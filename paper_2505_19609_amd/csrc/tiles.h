// LDS tiles shared by the attention kernels.
//
// A tile is 64 rows (keys, or queries in the dK/dV kernel) x D bf16, fetched by
// asynchronous buffer loads that write LDS directly (no data registers, no LDS
// store instructions, no address arithmetic in the vector ALU) and read back
// as MFMA operand fragments two ways:
//   * "rows":  A operand of a product that contracts over D       (16-byte reads)
//   * "cols":  A operand of a product that contracts over the rows (transposing
//              8-byte reads, ds_read_b64_tr_b16)
//
// Layout.  LDS has 64 banks of 4 bytes (a 256-byte line); a wave's 16-byte
// reads are served 16 lanes at a time and its 8-byte reads 32 lanes at a time,
// and a group is conflict-free when its 16-byte slots are distinct modulo 256
// bytes.  Rows are stored with 16 bytes of padding (row pitch D*2+16) and, within
// every group of 16 rows, in transposed 4x4 order (row r sits at position
// 4*(r%4) + (r/4)%4).  Then
//   * 16 consecutive rows at one column (operand reads) sit at 16 different
//     positions, hence 16 different slots, and
//   * 4 consecutive rows x 64 bytes (transposing reads) sit 4 positions apart,
//     hence again 16 different slots,
// and, unlike an XOR swizzle, every fragment address is ONE per-lane base plus
// a compile-time constant, so the hot loops spend no vector ALU work on LDS
// addresses (the VALU issue port is the scarce resource next to the MFMAs).
#pragma once

#include "mfma.h"

constexpr int TILE_ROWS = 64;

// nothing is scheduled across this point: pins the hand-made order of the steps
#define SB() __builtin_amdgcn_sched_barrier(0)

template <int D>
struct TileGeom {
    static constexpr int CH = D / 8;           // 16-byte chunks of payload per row
    static constexpr int SPR = CH + 1;         // 16-byte slots per row incl. padding
    static constexpr int ROWB = SPR * 16;      // row pitch in bytes
    static constexpr int SLOTS = TILE_ROWS * SPR;
    static constexpr int BYTES = SLOTS * 16;   // 17408 (D=128) / 9216 (D=64)
};

// position of row r inside the tile (an involution)
__device__ __forceinline__ int row_pos(int r) { return (r & ~15) | ((r & 3) << 2) | ((r >> 2) & 3); }

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// Per-lane fragment bases (two registers), lane = 32*h + n.
//   rows(t, b, ks):      rows 32*b + n of tile t, columns 16*ks + 8*h .. +7
//   cols(t, tt, kbg):    column 32*tt + n of rows 16*kbg + {4h..4h+3, 8+4h..8+4h+3},
//                        i.e. the rows that accumulator registers 8*(kbg%2)..+7
//                        of a 32x32 MFMA result stand for.
// The transposing read works on groups of 16 lanes: lane s of a group supplies
// the address of 4 consecutive columns of one row; lane l receives element l%4
// of the rows supplied by lanes l/4, l/4+4, l/4+8, l/4+12.
template <int D>
struct FragAddr {
    typedef TileGeom<D> G;
    int rm, tr;

    __device__ __forceinline__ void init(int lane)
    {
        const int n = lane & 31, h = lane >> 5;
        rm = row_pos(n) * G::ROWB + h * 16;
        const int grp = lane >> 4, s = lane & 15;
        // rows 4*(grp/2) + s/4 sit at positions 4*(s/4) + grp/2
        tr = (4 * (s >> 2) + (grp >> 1)) * G::ROWB + (2 * (grp & 1) + ((s & 3) >> 1)) * 16 + 8 * (s & 1);
    }
    __device__ __forceinline__ bf16x8 rows(const unsigned char *t, int b, int ks) const
    {
        return *(const bf16x8 *)(t + rm + b * (32 * G::ROWB) + ks * 32);
    }
    __device__ __forceinline__ bf16x8 cols(const unsigned char *t, int tt, int kbg) const
    {
        typedef s16x4 __attribute__((address_space(3))) * lds_ptr_t;
        const unsigned char *p = t + tr + kbg * (16 * G::ROWB) + tt * 64;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)p);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 2 * G::ROWB));  // rows +8
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, both);
    }
};

// ---------------------------------------------------------------------------
// Asynchronous fetch of 64-row tiles of one [rows, H, D] matrix restricted to one
// head.  One instruction makes a wave fill 64 consecutive 16-byte LDS slots (slot =
// M0 base + lane) from per-lane offsets, so the row permutation and the padding are
// applied on the global side: the lane that fills slot P fetches the chunk that
// belongs there (padding slots fetch a harmless duplicate).  The two instructions are
// written out (M0 <- LDS address; buffer load to LDS).  The compiler does not see these as
// writes to LDS, so operand reads of OTHER ring slots are not made to wait for
// a fetch in flight, whichever slot a run-time index selects; the kernels order
// a slot's fetch and its reads themselves (wait_vmem + workgroup barrier).
// ---------------------------------------------------------------------------
typedef int i32x4 __attribute__((ext_vector_type(4)));

// raw buffer descriptor words over `bytes` bytes at `base` (wave-uniform)
__device__ __forceinline__ i32x4 rsrc_words(const void *base, uint32_t bytes)
{
    const uint64_t p = (uint64_t)base;
    i32x4 r = {(int)__builtin_amdgcn_readfirstlane((uint32_t)p),
               (int)(__builtin_amdgcn_readfirstlane((uint32_t)(p >> 32)) & 0xffff),
               (int)__builtin_amdgcn_readfirstlane(bytes), 0x00020000};
    return r;
}

__device__ __forceinline__ uint32_t lds_addr(const void *p)
{
    typedef const unsigned char __attribute__((address_space(3))) * lds_cptr_t;
    return (uint32_t)(uintptr_t)(lds_cptr_t)p;
}

// 64 lanes x 16 bytes -> LDS [lds .. lds+1024); lane l fetches from base + voff + soff
__device__ __forceinline__ void dma_b128(i32x4 rsrc, uint32_t lds, int voff, int soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}
// 64 lanes x 4 bytes -> LDS [lds .. lds+256)
__device__ __forceinline__ void dma_b32(i32x4 rsrc, uint32_t lds, int voff, int soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :: "s"(lds), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}

// Tile loader for NWV wavefronts: wave w issues the 64-slot groups w, w+NWV, ...
// of the tile (17 groups at d=128, 9 at d=64), so every instruction runs with
// all lanes on and the only per-lane state is one byte offset per group.
template <int D, int NWV>
struct RingLoader {
    typedef TileGeom<D> G;
    static constexpr int GROUPS = G::SLOTS / 64;
    static constexpr int PER = (GROUPS + NWV - 1) / NWV;
    static_assert(G::SLOTS % 64 == 0, "tile slots must fill whole wave instructions");
    int voff[PER];
    uint32_t pitch;

    __device__ __forceinline__ void init(int lane, int wave, uint32_t row_pitch_bytes)
    {
        pitch = row_pitch_bytes;
#pragma unroll
        for (int x = 0; x < PER; ++x) {
            const int P = (x * NWV + wave) * 64 + lane;
            const int pos = P / G::SPR, c = P % G::SPR;
            voff[x] = row_pos(pos & 63) * (int)row_pitch_bytes + (c < G::CH ? c * 16 : 0);
        }
    }
    // descriptor over rows [0, valid_rows) of one head of a [rows, H, D] matrix
    __device__ __forceinline__ i32x4 rsrc(const uint16_t *row0_head, int valid_rows) const
    {
        return rsrc_words(row0_head, (uint32_t)(valid_rows - 1) * pitch + D * 2);
    }
    __device__ __forceinline__ void load(i32x4 r, uint32_t lds, int first_row, int wave) const
    {
        const int soff = (int)((uint32_t)first_row * pitch);  // below 2^32: checked when the plan is made
#pragma unroll
        for (int x = 0; x < PER; ++x)
            if (x * NWV + wave < GROUPS) dma_b128(r, lds + (x * NWV + wave) * 1024, voff[x], soff);
    }
};

// Wait until this wave's outstanding vector-memory loads (incl. loads to LDS) have landed.
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

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

// The same tile set as unrounded fp32 rows of a [rows, H, D] float tensor.
template <int TT>
__device__ __forceinline__ void store_rows_f32(float *dst, const f32x16 (&acc)[TT], int h)
{
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int vb = 0; vb < 4; ++vb)
            *(float4 *)(dst + 32 * tt + 8 * vb + 4 * h) =
                make_float4(acc[tt][4 * vb + 0], acc[tt][4 * vb + 1], acc[tt][4 * vb + 2], acc[tt][4 * vb + 3]);
}

// x + (x of the lane 32 away).  Written out with the operands copied first: given one
// value for both operands, the swap builtin returns its first result twice.
__device__ __forceinline__ float add_other_half(float x)
{
    float r, t;
    asm volatile("v_mov_b32 %0, %2\n\tv_mov_b32 %1, %2\n\ts_nop 1\n\t"
                 "v_permlane32_swap_b32 %0, %1\n\tv_add_f32 %0, %0, %1"
                 : "=&v"(r), "=&v"(t) : "v"(x));
    return r;
}

template <int N>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[N])
{
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
}
