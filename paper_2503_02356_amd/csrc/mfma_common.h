// Device-side helpers shared by the bf16 MFMA kernels (gfx950).
//
// MFMA 32x32x16 bf16 operand layout (lane l of a 64-wide wavefront, half = l / 32):
//   A (M x K): lane holds row  m = l % 32, k = 8*half + 0..7        (bf16x8)
//   B (K x N): lane holds col  n = l % 32, k = 8*half + 0..7        (bf16x8)
//   C/D (M x N, fp32x16): lane holds col n = l % 32, register i <-> row (i/4)*8 + 4*half + i%4
//
// ds_read_tr16_b64 (transposing LDS read): inside each block of 16 lanes, lane r supplies the address
// of 4 consecutive 16-bit elements; the 16x4 elements are handed out so that lane i receives
// element (i % 4) of the rows supplied by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4.  With lane r
// pointing at mem[k0 + r/4][n0 + 4*(r%4)] (a 4 x 16 block of a row-major matrix), lane i therefore
// gets mem[k0 + 0..3][n0 + i]: four consecutive k for one n -- half of an MFMA operand whose
// contraction index runs along the matrix rows.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "chunkflow.h"

namespace cf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

#define CF_LDS __attribute__((address_space(3)))

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Two transposing reads, 8 rows apart... the caller passes both addresses; result is one bf16x8 operand.
__device__ __forceinline__ bf16x8 lds_read_tr_pair(const char *lo_addr, const char *hi_addr)
{
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CF_LDS s16x4 *)lo_addr);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((CF_LDS s16x4 *)hi_addr);
    s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ bf16x8 lds_read_b128(const char *addr)
{
    return *(const bf16x8 *)addr;
}

// Packs 8 fp32 values into a bf16x8 (round to nearest even; v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3, float a4, float a5, float a6,
                                        float a7)
{
    bf16x8 r;
    r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
    r[4] = (__bf16)a4; r[5] = (__bf16)a5; r[6] = (__bf16)a6; r[7] = (__bf16)a7;
    return r;
}

// Swizzled LDS tile with 256-byte rows (128 bf16) and no padding: the 16-byte unit u of row r lives at
// unit u ^ swz(r).  LDS has 64 four-byte banks; a 16-byte row read (ds_read_b128) is served 16 lanes per
// clock and a transposing 8-byte read (ds_read_b64_tr_b16) 32 lanes per clock.  swz() maps 16 consecutive
// rows to 16 different units (row reads of one column by 16 rows are conflict free) AND gives the 4
// consecutive rows of a transposing read 4 different groups of 4 units (those are conflict free too).
__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
__device__ __forceinline__ int tile_off(int row, int unit) { return row * 256 + ((unit ^ swz(row)) << 4); }

// Lane-constant LDS byte offsets into a swizzled tile, computed once per kernel (the XOR of the swizzle
// cannot be folded into an instruction's immediate offset, so every distinct unit needs its own register;
// keeping them in 16 registers beats recomputing them for each of the ~100 LDS reads per tile).
//
//  row_unit[ks]  operand rows read with ds_read_b128 (MFMA row/col = tile row, contraction along the tile
//                row): offset of (row = lane % 32, logical unit 2*ks + half).  A 32-row block further down
//                the tile adds 32*256 bytes (swz() has period 16 rows).
//  tr_lo[db], tr_hi[db]
//                operands read with the transposing read (contraction along the tile's ROWS, MFMA
//                row/col = tile column 32*db + lane % 32): offsets of the two 4-row reads that make one
//                bf16x8 operand, for contraction rows 4*half + {0..3 by lane group} and 8 rows further.
//                32 (16) rows further down the tile add 32*256 (16*256) bytes.
struct LaneOffsets {
    int row_unit[8];
    int tr_lo[4], tr_hi[4];
};
__device__ __forceinline__ LaneOffsets lane_offsets()
{
    const int lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31, r16 = lane & 15, blk = (lane >> 4) & 1;
    LaneOffsets o;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) o.row_unit[ks] = tile_off(col, 2 * ks + half);
    const int r_lo = 4 * half + (r16 >> 2), u0 = 2 * blk + ((r16 >> 1) & 1), sub = 8 * (r16 & 1);
#pragma unroll
    for (int db = 0; db < 4; ++db) {
        o.tr_lo[db] = tile_off(r_lo, 4 * db + u0) + sub;
        o.tr_hi[db] = tile_off(r_lo + 8, 4 * db + u0) + sub;
    }
    return o;
}

// Index of this wavefront inside its workgroup, as a value the compiler knows to be wave-uniform.
__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// Direct global -> LDS copy of a swizzled tile of ROWS x 256 bytes by a workgroup of WAVES wavefronts
// (buffer_load_dwordx4 ... lds: no staging registers; lane i of one instruction lands at LDS base + 16*i, so
// one instruction fills 4 tile rows and the swizzle is applied on the global side: the lane that fills
// physical unit u' of row r fetches logical unit u' ^ swz(r)).
// A tile takes ROWS / (4 * WAVES) instructions per wavefront (PARTS); each costs the issuing wavefront some 30-45 clocks
// wherever it is placed (measured), so they are simply issued together at the start of a tile.
// Addressing is the buffer form on purpose: the tile's first row is a wave-uniform pointer that becomes the
// base of a buffer descriptor (scalar arithmetic), the lane's place inside a tile is ONE register computed
// at init, and a part adds a scalar offset, so a full tile costs no vector address arithmetic at all.  Only
// a ragged tile (rows beyond last_row, relative to src, re-read last_row; the caller masks them) computes
// clamped per-lane offsets.  The descriptor's size field is left at its maximum: nothing relies on the
// hardware's out-of-range behaviour.
// Completion is tracked by vmcnt: wait_lds_dma() before the barrier that publishes the tile.
template <int ROWS, int WAVES = 4>
struct TileDma {
    static constexpr int PARTS = ROWS / (4 * WAVES);
    static_assert(PARTS >= 1 && (4 * WAVES) % 16 == 0, "a part must cover whole swizzle periods");
    unsigned row_bytes, unit16;   // unit16: byte offset of this lane's 16-byte unit inside its row (same for all parts)
    int r0;                       // this lane's row in part 0; part c adds 4 * WAVES rows
    int wv;                       // index of this wavefront among the copying ones
    unsigned lane_off;            // r0 * row_bytes + unit16: this lane's offset in part 0 of a full tile

    // wave: index of the calling wavefront among the WAVES that copy (wave-uniform)
    __device__ __forceinline__ void init(int64_t row_bytes_, int wave)
    {
        const int lane = threadIdx.x & 63;
        row_bytes = (unsigned)row_bytes_;
        wv = wave;
        r0 = 4 * wave + (lane >> 4);
        unit16 = ((lane & 15) ^ swz(r0)) * 16;       // swz() has period 16 rows
        lane_off = (unsigned)r0 * row_bytes + unit16;
    }
    __device__ __forceinline__ void init(int64_t row_bytes_) { init(row_bytes_, wave_id()); }
    __device__ __forceinline__ CF_LDS void *part_dst(char *lds_tile, int c) const { return (CF_LDS void *)(lds_tile + (c * WAVES + wv) * 1024); }
    __device__ __forceinline__ static __amdgpu_buffer_rsrc_t descriptor(const char *src)
    {
        return __builtin_amdgcn_make_buffer_rsrc((void *)src, 0, -1, 0x00020000);
    }
    __device__ __forceinline__ void full_part(__amdgpu_buffer_rsrc_t rsrc, char *lds_tile, int c) const
    {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, part_dst(lds_tile, c), 16, (int)lane_off, (int)(4 * WAVES * c * row_bytes), 0, 0);
    }
    __device__ __forceinline__ void ragged_part(__amdgpu_buffer_rsrc_t rsrc, int last_row, char *lds_tile, int c) const
    {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, part_dst(lds_tile, c), 16,
                                                 (int)((unsigned)min(r0 + 4 * WAVES * c, last_row) * row_bytes + unit16), 0, 0, 0);
    }
    // last_row is wave-uniform, so the branches below are scalar ones.
    __device__ __forceinline__ void issue_part(const char *src, int last_row, char *lds_tile, int c) const
    {
        if (last_row >= ROWS - 1) full_part(descriptor(src), lds_tile, c);
        else ragged_part(descriptor(src), last_row, lds_tile, c);
    }
    __device__ __forceinline__ void issue(const char *src, int last_row, char *lds_tile) const
    {
        const __amdgpu_buffer_rsrc_t rsrc = descriptor(src);
        if (last_row >= ROWS - 1) {
#pragma unroll
            for (int c = 0; c < PARTS; ++c) full_part(rsrc, lds_tile, c);
        } else {
#pragma unroll
            for (int c = 0; c < PARTS; ++c) ragged_part(rsrc, last_row, lds_tile, c);
        }
    }
};
// Makes a pointer / an int that is the same in every lane known as such to the compiler.
template <typename T>
__device__ __forceinline__ T *uniform(T *p)
{
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (T *)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ void wait_lds_dma() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)

// The 128-row query tile of workgroup rank `rank` from the caller's table (cf_attn_q_tiles: heaviest tile first,
// each record carries its segment's bounds): one uniform 32-byte read instead of the search of locate_tile.
struct QTile {
    int tile_in_seg, q_begin, q_len, k_begin, k_len;
};
__device__ __forceinline__ QTile read_q_tile(const cf_q_tile *table, int rank)
{
    const i32x4 *rec = (const i32x4 *)(table + rank);
    const i32x4 a = rec[0], b = rec[1];
    return QTile{uniform(b[0]), uniform(a[0]), uniform(a[1]), uniform(a[2]), uniform(a[3])};
}

// Stores a wavefront's 32 x 128 block of bf16 results (computed transposed: a lane owns one ROW, register group
// (j, g4) of acc holds its 4 consecutive d starting at 32*j + 8*g4 + 4*half) to global rows of 256 bytes.
// A direct store would write 8-byte pieces of 32 different rows per instruction (64 cache lines touched per
// instruction, 16 instructions); instead the block is turned around in `scratch` (this wavefront's own
// 32 x 272 bytes of LDS, free at that point) and leaves as 8 instructions that each write 4 whole rows.
//   row_ptr(r): global address of row r of the block (r = 0..31), rows >= rows_valid are not written
constexpr int kRowScratchStride = 272;          // 256 + 16: keeps 16-byte alignment, spreads rows over banks
constexpr int kRowScratchBytes = 32 * kRowScratchStride;
template <typename RowPtr>
__device__ __forceinline__ void store_rows_bf16(const f32x16 (&acc)[4], float scale, char *scratch, int rows_valid,
                                                RowPtr row_ptr)
{
    const int lane = threadIdx.x & 63, half = lane >> 5, col = lane & 31;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (__bf16)(acc[j][g4 * 4 + e] * scale);
            *(bf16x4 *)(scratch + col * kRowScratchStride + (j * 32 + g4 * 8 + half * 4) * 2) = w;
        }
    __builtin_amdgcn_wave_barrier();
    bf16x8 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = *(const bf16x8 *)(scratch + (4 * i + (lane >> 4)) * kRowScratchStride + (lane & 15) * 16);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = 4 * i + (lane >> 4);
        if (r < rows_valid) *(bf16x8 *)(row_ptr(r) + (lane & 15) * 16) = v[i];
    }
}

// Lane l and lane l ^ 32 combine a value without going through LDS: v_permlane32_swap with both operands = x
// returns (x of the lower half, x of the upper half) in every lane (checked on the device with a probe).
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float max_with_other_half(float x)
{
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_with_other_half(float x)
{
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Finds the tile a workgroup owns.  Tiles of `tile` rows are counted per segment over cu[0..n_seg]
// and numbered from the LAST tile of the LAST segment backwards (the later tiles of a segment see more
// keys, so the heaviest tiles get the lowest ranks and start first).  Every lane of every wavefront
// computes the same answer.  Returns false if rank >= number of tiles.
// The lanes that scan the segment list load its bounds in BOTH lists (cu: the list the tiles are counted
// over, cu_other: the other one), and the winner's values are handed out by lane reads: the caller gets
// the segment's four bounds without a second, dependent round of loads.
struct TileLocation {
    int seg, tile_in_seg;
    int begin, len;               // of the segment in cu
    int other_begin, other_len;   // of the segment in cu_other
};
__device__ __forceinline__ bool locate_tile(const int32_t *cu, const int32_t *cu_other, int n_seg, int tile, int rank,
                                            TileLocation &out)
{
    const int lane = threadIdx.x & 63;
    for (int base = 0; base < n_seg; base += 64) {
        const int gi = n_seg - 1 - (base + lane);
        int cnt = 0, b0 = 0, b1 = 0, o0 = 0, o1 = 0;
        if (gi >= 0) {
            b0 = cu[gi];
            b1 = cu[gi + 1];
            o0 = cu_other[gi];
            o1 = cu_other[gi + 1];
            cnt = (b1 - b0 + tile - 1) / tile;
        }
        int inc = cnt;
        for (int o = 1; o < 64; o <<= 1) {
            const int t = __shfl_up(inc, o);
            if (lane >= o) inc += t;
        }
        const int total = __shfl(inc, 63);
        if (rank < total) {
            const unsigned long long ball = __ballot(inc > rank);
            const int first = __ffsll((long long)ball) - 1;
            const int exc = __shfl(inc - cnt, first);
            const int c = __shfl(cnt, first);
            out.seg = __builtin_amdgcn_readfirstlane(n_seg - 1 - (base + first));
            out.tile_in_seg = __builtin_amdgcn_readfirstlane(c - 1 - (rank - exc));
            out.begin = __builtin_amdgcn_readfirstlane(__shfl(b0, first));
            out.len = __builtin_amdgcn_readfirstlane(__shfl(b1 - b0, first));
            out.other_begin = __builtin_amdgcn_readfirstlane(__shfl(o0, first));
            out.other_len = __builtin_amdgcn_readfirstlane(__shfl(o1 - o0, first));
            return true;
        }
        rank -= total;
    }
    return false;
}

}  // namespace cf
