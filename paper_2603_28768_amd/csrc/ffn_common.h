// Pieces shared by the grouped-GEMM kernels: the tile list walk and small device helpers.
#pragma once

#include <algorithm>

#include "kernels.h"

namespace craft {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

struct Tile {
    int32_t slot;      // local slot index
    int32_t m0;        // first row inside the slot
    int32_t rows;      // valid rows in this tile
    int32_t n0;        // first output column
    int32_t pos0;      // global dispatch position of the slot's first row
};

// Flattened work item w -> tile.  nt = column tiles per slot, bm/bn tile extents.
static __device__ __forceinline__ Tile decode_tile(const FfnArgs &a, int64_t w, int32_t nt, int32_t bm,
                                            int32_t bn) {
    const int32_t qn = (int32_t)(w / nt);
    int32_t lo = 0, hi = a.nslots;                 // find s: mt_start[s] <= qn < mt_start[s+1]
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (a.mt_start[mid] <= qn) lo = mid; else hi = mid;
    }
    const int32_t mt_first = a.mt_start[lo];
    const int32_t mts = a.mt_start[lo + 1] - mt_first;
    const int32_t s = a.order[lo];             // the list is ordered busiest slot first
    const int32_t rem = (int32_t)(w - (int64_t)mt_first * nt);
    Tile t;
    t.slot = s;
    t.m0 = (rem % mts) * bm;
    t.n0 = (rem / mts) * bn;
    t.pos0 = a.slot_off[a.s_lo + s];
    t.rows = min(bm, a.slot_off[a.s_lo + s + 1] - t.pos0 - t.m0);
    return t;
}

// The same walk over a copy of the three small tables held in LDS (loaded once per
// workgroup), which takes the chain of dependent global reads out of every tile's start.
struct TileTables {
    static constexpr int kMaxSlots = 256;
    int32_t mt_start[kMaxSlots + 1];
    int32_t order[kMaxSlots];
    int32_t slot_off[kMaxSlots + 1];      // offsets of the rank's slots, busiest-first order undone
};
static __device__ __forceinline__ void load_tile_tables(const FfnArgs &a, TileTables &tt) {
    for (int i = threadIdx.x; i <= a.nslots; i += blockDim.x) {
        tt.mt_start[i] = a.mt_start[i];
        tt.slot_off[i] = a.slot_off[a.s_lo + i];
        if (i < a.nslots) tt.order[i] = a.order[i];
    }
    __syncthreads();
}
static __device__ __forceinline__ Tile decode_tile(const FfnArgs &a, const TileTables &tt, int64_t w,
                                                   int32_t nt, int32_t bm, int32_t bn) {
    const int32_t qn = (int32_t)(w / nt);
    int32_t lo = 0, hi = a.nslots;
    while (hi - lo > 1) {
        const int32_t mid = (lo + hi) >> 1;
        if (tt.mt_start[mid] <= qn) lo = mid; else hi = mid;
    }
    const int32_t mt_first = tt.mt_start[lo];
    const int32_t mts = tt.mt_start[lo + 1] - mt_first;
    const int32_t s = tt.order[lo];
    const int32_t rem = (int32_t)(w - (int64_t)mt_first * nt);
    Tile t;
    t.slot = s;
    t.m0 = (rem % mts) * bm;
    t.n0 = (rem / mts) * bn;
    t.pos0 = tt.slot_off[s];
    t.rows = min(bm, tt.slot_off[s + 1] - t.pos0 - t.m0);
    return t;
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

}  // namespace craft
