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
    // the same fragment of the first 32 rows of a tile-shaped region given by its LDS address
    __device__ __forceinline__ bf16x8 rows_at(uint32_t region, int ks) const
    {
        typedef bf16x8 __attribute__((address_space(3))) * lds_frag_t;
        return *(lds_frag_t)(uintptr_t)(region + rm + ks * 32);
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

// ---------------------------------------------------------------------------
// Per-wave staging of a 32-row block of one head of a [rows, H, D] matrix.
//
// A lane of a 32x32 MFMA owns one ROW of such a block (B operand: 16 bytes of it per
// k-step; result: 8 bytes per four accumulator registers).  Loading or storing the block
// straight from that layout touches 32 rows per instruction, 16 or 8 bytes of each: 64
// separate cache requests per instruction, and the 8 to 24 such instructions per lane at
// the start and end of a work item kept the address path busy for 3 to 14 us per item.
// Here the wave moves the block in whole rows instead (64 lanes x 16 bytes = 4 rows at
// D = 128, 8 rows at D = 64 per instruction) and turns it in a private LDS region laid out
// like the first half of a tile (32 rows, same pitch and row permutation), so the operand
// fragments come back through FragAddr::rows_at and results go in by quads.  LDS
// instructions of one wave execute in order, so the region needs no barrier between its
// write and read; the caller makes sure no other wave uses the same bytes as a tile
// meanwhile.  Regions are given as 32-bit LDS addresses.
// ---------------------------------------------------------------------------
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x4 __attribute__((address_space(3))) * lds_u4_t;
typedef u32x2 __attribute__((address_space(3))) * lds_u2_t;

template <int D>
struct WaveStage {
    typedef TileGeom<D> G;
    static constexpr int BYTES = 32 * G::ROWB;  // 8704 (D=128) / 4608 (D=64)
    static constexpr int N = 32 * G::CH / 64;   // whole-row instructions per block: 8 / 4
    static constexpr int RPI = 64 / G::CH;      // rows per instruction: 4 / 8
    int r_in, c16;                              // this lane's row inside an instruction's rows; its byte column

    __device__ __forceinline__ void init(int lane)
    {
        r_in = lane / G::CH;
        c16 = (lane % G::CH) * 16;
    }
    // rows first .. first+31 of a matrix of `rows` >= 1 rows (row index clamped to the last one);
    // `base` points at row 0, column 0 of the head
    __device__ __forceinline__ void load(u32x4 (&v)[N], const uint16_t *base, uint32_t pitch_bytes, int first,
                                         int rows) const
    {
        const unsigned char *b = (const unsigned char *)base + c16;
#pragma unroll
        for (int j = 0; j < N; ++j)
            v[j] = *(const u32x4 *)(b + (size_t)min(first + j * RPI + r_in, rows - 1) * pitch_bytes);
    }
    __device__ __forceinline__ void put(uint32_t region, const u32x4 (&v)[N]) const
    {
#pragma unroll
        for (int j = 0; j < N; ++j)
            *(lds_u4_t)(uintptr_t)(region + row_pos(j * RPI + r_in) * G::ROWB + c16) = v[j];
    }
    // 32 (d) x 32 (row) accumulator tiles of this lane's row n (half h), scaled, as bf16
    template <int TT>
    __device__ __forceinline__ void put_acc(uint32_t region, const f32x16 (&acc)[TT], float mul, int n, int h) const
    {
        const uint32_t a = region + row_pos(n) * G::ROWB + 8 * h;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int vb = 0; vb < 4; ++vb) {
                u32x2 w;
                w.x = pack_bf16(acc[tt][4 * vb + 0] * mul, acc[tt][4 * vb + 1] * mul);
                w.y = pack_bf16(acc[tt][4 * vb + 2] * mul, acc[tt][4 * vb + 3] * mul);
                *(lds_u2_t)(uintptr_t)(a + 64 * tt + 16 * vb) = w;
            }
    }
    // the staged block to rows first .. first+31 of the matrix (those below `rows`), whole rows per instruction
    __device__ __forceinline__ void store(uint32_t region, uint16_t *base, uint32_t pitch_bytes, int first,
                                          int rows) const
    {
        unsigned char *b = (unsigned char *)base + c16;
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const u32x4 w = *(lds_u4_t)(uintptr_t)(region + row_pos(j * RPI + r_in) * G::ROWB + c16);
            const int r = first + j * RPI + r_in;
            if (r < rows) *(u32x4 *)(b + (size_t)r * pitch_bytes) = w;
        }
    }
};

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
