// Pieces shared by the grouped-GEMM kernels: the tile list walk and small device helpers.
#pragma once

#include <algorithm>

#include "kernels.h"

namespace craft {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

struct Tile {
    int32_t slot;      // local slot index
    int32_t m0;        // first row inside the slot
    int32_t rows;      // valid rows in this tile
    int32_t n0;        // first output column
    int32_t pos0;      // global dispatch position of the slot's first row
    int32_t mtile;     // index of the row-tile in the list of all row-tiles of the busy slots
    int32_t single;    // 1 when this is the slot's only row-tile (nobody else reads its weights)
};

// Flattened work item w -> tile.  nt = column tiles per slot, bn = columns per tile.
// mt_start[p] = row-tiles before position p of the busiest-first slot order.  A slot's rows
// are cut into F 32-row fragments and m = ceil(F / f) row-tiles, either f fragments each with
// a remainder at the end, or shared as evenly as whole fragments allow (row-tile i takes
// fragments floor(i F / m) .. floor((i+1) F / m)); the launch says which.
//
// Inside a slot the m x nt tiles are listed column by column, or (`blocked`) block by block:
// bands of kBandRows row-tiles, a band cut into blocks of kBlockCols column tiles, a block
// column by column.  A run of consecutive list entries, which is what runs at one time (tiles
// are handed out in list order), is then a compact rectangle of tiles that needs few row-tiles
// of activations and few column tiles of weights between them, where a run of the column
// order needs every row-tile of the slot for each of its columns.  At T = 32768 (five rounds of
// tiles) the step is 4 % faster with 8 x 8 blocks than column by column (4 x 8, 8 x 4: 3 %;
// 2 x 16, 16 x 16, 1 x 8: 2 %); the packed kernels use the block order for launches of more
// than two rounds.
constexpr int kBandRows = 8;
constexpr int kBlockCols = 8;
struct TileTables {
    static constexpr int kMaxSlots = 256;
    int32_t mt_start[kMaxSlots + 1];
    int32_t order[kMaxSlots];
    int32_t slot_off[kMaxSlots + 1];      // offsets of the rank's slots, busiest-first order undone
};
static __device__ __forceinline__ void load_tile_tables(const FfnArgs &a, const int32_t *mt_start,
                                                        TileTables &tt) {
    for (int i = threadIdx.x; i <= a.nslots; i += blockDim.x) {
        tt.mt_start[i] = mt_start[i];
        tt.slot_off[i] = a.slot_off[a.s_lo + i];
        if (i < a.nslots) tt.order[i] = a.order[i];
    }
    __syncthreads();
}
// MT, ORD, OFF: the three tables, in global memory or in a workgroup's LDS copy
// fmax > 0: row-tiles of fmax fragments and a remainder; fmax < 0: |fmax| at most, shared evenly
template <typename MT, typename ORD, typename OFF>
static __device__ __forceinline__ Tile decode_tile_in(int32_t nslots, const MT &mt_start, const ORD &order,
                                                      const OFF &slot_off, int64_t w, int32_t nt, int32_t bn,
                                                      int32_t fmax, bool blocked) {
    const int32_t qn = (int32_t)(w / nt);
    int32_t lo = 0, hi = nslots;                   // find p: mt_start[p] <= qn < mt_start[p+1]
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (mt_start[mid] <= qn) lo = mid; else hi = mid;
    }
    const int32_t mt_first = mt_start[lo];
    const int32_t mts = mt_start[lo + 1] - mt_first;
    const int32_t s = order[lo];
    const int32_t rem = (int32_t)(w - (int64_t)mt_first * nt);
    const int32_t band = blocked ? kBandRows : mts;             // column by column: one band, one column per block
    const int32_t bcols = blocked ? kBlockCols : 1;
    const int32_t r0 = rem / (band * nt) * band;                // first row-tile of the band
    const int32_t rj = min(band, mts - r0);                     // row-tiles in this band
    const int32_t in_band = rem - r0 * nt;
    const int32_t cb = in_band / (rj * bcols);                  // block of columns inside the band
    const int32_t in_block = in_band - cb * rj * bcols;
    const int32_t i = r0 + in_block % rj;
    const int32_t col = cb * bcols + in_block / rj;
    Tile t;
    t.slot = s;
    t.pos0 = slot_off[s];
    const int32_t slot_rows = slot_off[s + 1] - t.pos0;
    const int32_t frags = (slot_rows + 31) >> 5;
    const int32_t f0 = fmax > 0 ? i * fmax : (int32_t)((int64_t)i * frags / mts);
    const int32_t f1 = fmax > 0 ? min(f0 + fmax, frags) : (int32_t)((int64_t)(i + 1) * frags / mts);
    t.m0 = f0 * 32;
    t.rows = min(f1 * 32, slot_rows) - t.m0;
    t.n0 = col * bn;
    t.mtile = mt_first + i;
    t.single = mts == 1 ? 1 : 0;
    return t;
}
static __device__ __forceinline__ Tile decode_tile(const FfnArgs &a, const int32_t *mt_start, int64_t w,
                                                   int32_t nt, int32_t bn, int32_t fmax, bool blocked = false) {
    return decode_tile_in(a.nslots, mt_start, a.order, a.slot_off + a.s_lo, w, nt, bn, fmax, blocked);
}
static __device__ __forceinline__ Tile decode_tile(const FfnArgs &a, const TileTables &tt, int64_t w,
                                                   int32_t nt, int32_t bn, int32_t fmax, bool blocked = false) {
    return decode_tile_in(a.nslots, tt.mt_start, tt.order, tt.slot_off, w, nt, bn, fmax, blocked);
}

// Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous run of the
// tile list per sweep so that tiles sharing weights meet in one L2.
static __device__ __forceinline__ int64_t xcd_major_id() {
    const int64_t g = gridDim.x, b = blockIdx.x;
    return (b % 8) * (g / 8) + b / 8;
}

static __device__ __forceinline__ uint32_t bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
static __device__ __forceinline__ float silu(float g) { return g / (1.0f + __expf(-g)); }
// The same with the hardware reciprocal (1 ulp) instead of a correctly rounded division: the
// result is rounded to bf16 right after.
static __device__ __forceinline__ float silu_fast(float g) {
    return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g));
}
// Two fp32 values to a pair of bf16 (round to nearest even) in one 32-bit word, low half first:
// a single v_cvt_pk_bf16_f32 on gfx950.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
static __device__ __forceinline__ uint32_t bf16_pair(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

}  // namespace craft
