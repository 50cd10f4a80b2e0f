// Internal launcher interface between the host API (forward.cpp) and the HIP kernels.
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

#include "plan_internal.h"

namespace craft {

// Tokens handled by one workgroup of the routing and dispatch kernels.  Ranks of
// assignments inside a block are taken from a 32-bit token mask per expert.
constexpr int kTokPerBlock = 32;
// Blocks of tokens whose per-expert counts one workgroup of the scan kernel prefixes.
constexpr int kScanChunk = 256;

// Control words at the start of the workspace.
enum { CTRL_TICKET = 0, CTRL_ROWS = 1, CTRL_OVERFLOW = 2, CTRL_MTILES = 3,
       CTRL_HOT_SLOTS = 6,                         // slots of the rank with more than kColdRows rows
       CTRL_LIVE_SLOTS = 7,                        // slots of the rank with any rows
       CTRL_RIDERS_GATEUP = 8, CTRL_RIDERS_DOWN = 9,   // rider units carried by the busy slots' tiles, per GEMM
       CTRL_COLD2_SLOTS = 10,                      // cold slots with two fragments (33 .. kColdRows rows)
       CTRL_WORK_GATEUP = 4, CTRL_WORK_DOWN = 5,   // dynamic tile counters of the two GEMMs
       CTRL_WORDS = 16 };

// A slot with at most this many rows is "cold": its tiles do next to no matrix work and are
// bound by streaming the weights.  The packed FFN cuts their column tiles in half (twice as
// many, half as long), because what the tail of a launch costs is the length of a cold tile
// and the aggregate weight bandwidth grows with the number of CUs streaming at once.
constexpr int kColdRows = 64;

// Riders.  During a tile of a busy slot the CU's matrix pipeline is busy and HBM is not;
// during a cold slot's tile it is the other way round.  So a tile of a busy slot carries a
// "rider unit" along: one 32-row fragment of a cold slot against half a column tile of that
// slot's weights (one column group per wave), streamed through a second weight ring and
// costing four more MFMAs of 16 x 16 x 32 per 32-wide step.  Half a tile, not a whole one,
// because a CU's vector memory path (64 bytes per clock) is already two-thirds used by the
// tile's own operands.
// The units of the cold slots, in busiest-first order (two-fragment slots first), go to the
// tiles of the list one each, from the first tile on: unit u rides on tile u.  A two-fragment
// slot is carried whole or not at all.  Tiles of more than kRiderHostFrags fragments have no
// registers left for a rider: a launch with taller tiles carries none.
constexpr int kRiderHostFrags = 7;

// Most 32-row fragments a row-tile of the grouped GEMMs may have (the tile table is built for
// a height chosen per launch, up to these).
constexpr int kFragsBf16 = 4;      // LDS-staged bf16 kernels (row-major weights): 128 rows
constexpr int kFragsPacked = 8;    // weight-streaming bf16 kernels (packed weights): 256 rows
constexpr int kFragsF32 = 1;
constexpr int kBM_packed = kFragsPacked * 32;

struct RouterArgs {
    int32_t dtype;
    const void *x;            // [T][H]
    const void *w;            // [E][H] gate weights
    int64_t T;
    int32_t H, E;
    float *logits;            // [T][E]
    int32_t num_cu;
    float *part;              // [nsplit][T][E] partial scores when the contraction is split; may be null
    int32_t nsplit;           // set by the launcher
};
hipError_t launch_router_logits(const RouterArgs &a, hipStream_t s);
void router_logits_shape(int64_t T, int32_t H, int32_t E, int32_t num_cu, bool workspace, int *nxf, int *nsplit);

struct RouteArgs {
    const float *logits;
    int64_t T;
    int32_t E, k, renorm;
    int32_t *ids;       // [T][k]
    float *w;           // [T][k]
    uint8_t *lrank;     // [T][k] rank of the assignment among same-expert ones of its block; may be null
    int32_t *hist;      // [NB][E] per-block expert counts; may be null
    int32_t *ctrl;      // control words to clear; may be null
};
hipError_t launch_route(const RouteArgs &a, hipStream_t s);

struct ScanArgs {
    int32_t *hist;            // [NB][E] in: counts per block; out: exclusive prefix over the blocks of a chunk
    int32_t *chunk_tot;       // [chunks][E] totals of the chunks (scratch; more than one chunk only)
    int32_t *chunk_base;      // [chunks][E] out: sum of the earlier chunks' totals
    int32_t NB, E;
    const int32_t *tables;    // device tables of this (layer, rank)
    int32_t S, s_lo, s_hi;
    int64_t max_rows;
    int32_t *counts;          // [E]
    int32_t *slot_cnt;        // [S]
    int32_t *slot_off;        // [S+1]
    int32_t *ctrl;
    int32_t *user_counts, *user_slot_cnt, *user_slot_off;   // optional copies
};
hipError_t launch_scan(const ScanArgs &a, hipStream_t s);

struct DispatchArgs {
    const int32_t *ids;
    const uint8_t *lrank;
    const int32_t *base;      // [NB][E] prefixes inside a chunk of blocks
    const int32_t *chunk_base; // [chunks][E] on top of them; null when there is one chunk
    int64_t T;
    int32_t k, E;
    const int32_t *tables;
    const int32_t *slot_off;
    int32_t *dest, *src;
    int32_t *user_dest, *user_src;
    // for the extra workgroup that builds the tile tables of the grouped GEMMs
    const int32_t *slot_cnt;  // [S] rows per slot
    int32_t s_lo, s_hi;       // the rank's slots
    int32_t frags_gu, frags_dn;   // most 32-row fragments per row-tile, gate/up and down GEMM (sign: see FfnArgs)
    int32_t nt_gu, nt_dn;     // column tiles per slot of the two packed GEMMs; 0: no riders
    int32_t *mt_start;        // [2][s_hi - s_lo + 1] row-tile prefix over the rank's slots, busiest slot
                              // first: for the gate/up GEMM, then for the down GEMM
    int32_t *order;           // [s_hi - s_lo] local slot at each position of that order
    int32_t *ctrl;
};
hipError_t launch_dispatch(const DispatchArgs &a, hipStream_t s);

struct FfnArgs {
    int32_t dtype;
    int32_t H, I, k;
    int32_t s_lo, nslots;
    const void *x;                 // [T][H]
    const int32_t *src;            // [A]
    const int32_t *slot_off;       // [S+1]
    const int32_t *mt_start;       // [2][nslots+1]: gate/up, down
    const int32_t *order;          // [nslots]
    int32_t *ctrl;
    const void *const *w_gate, *const *w_up, *const *w_down;   // row-major weights per slot
    const void *const *wp_gateup, *const *wp_down;             // fragment-packed weights per slot
    void *act;                     // [max_rows][I] SwiGLU activations
    void *y;                       // [max_rows][H]
    int64_t max_rows;
    int32_t num_cu;
    int32_t w8;                    // packed weights are E4M3 codes with row scales behind the stream
    int32_t frags_gu, frags_dn;    // most 32-row fragments per row-tile the tile tables were built for;
                                   // negative: fragments shared evenly among a slot's row-tiles
};
hipError_t launch_gateup(const FfnArgs &a, hipStream_t s);
hipError_t launch_down(const FfnArgs &a, hipStream_t s);
hipError_t launch_gateup_packed(const FfnArgs &a, hipStream_t s);
hipError_t launch_down_packed(const FfnArgs &a, hipStream_t s);
void packed_sizes(int32_t H, int32_t I, size_t *gateup_bytes, size_t *down_bytes);
hipError_t launch_pack(int32_t H, int32_t I, const void *wg, const void *wu, const void *wd,
                       void *pgu, void *pdn, hipStream_t s);
void packed_sizes_e4m3(int32_t H, int32_t I, size_t *gateup_bytes, size_t *down_bytes);
hipError_t launch_quantize_e4m3(const void *w, int64_t rows, int32_t K, uint8_t *codes, float *scale,
                                hipStream_t s);
hipError_t launch_pack_e4m3(int32_t H, int32_t I, const uint8_t *cg, const uint8_t *cu, const uint8_t *cd,
                            const float *sg, const float *su, const float *sd, void *pgu, void *pdn,
                            hipStream_t s);

struct CombineArgs {
    int32_t dtype;
    int64_t T;
    int32_t k, H;
    const void *y;
    const int32_t *dest;
    const float *w;
    const int32_t *slot_off;
    int32_t s_lo, s_hi;
    const int32_t *ctrl;
    void *out;
};
hipError_t launch_combine(const CombineArgs &a, hipStream_t s);

struct LoadArgs {
    const int32_t *ids;       // [L][T][k]
    int32_t L, k, E;
    int64_t T, batch_tokens, B;
    int64_t *counts;          // [B][L][E]
};
hipError_t launch_expert_load(const LoadArgs &a, hipStream_t s);
hipError_t launch_probe_copy(const void *src, void *dst, int64_t bytes, int32_t num_cu, hipStream_t s);
hipError_t launch_probe_read(const void *src, int64_t bytes, int32_t passes, int32_t blocks, uint32_t *sink,
                             hipStream_t s);
hipError_t launch_probe_mfma(int32_t blocks, int32_t iters, float *sink, hipStream_t s);
hipError_t launch_probe_mfma_operands(int32_t shape, int32_t data, int32_t blocks, int32_t iters, float *sink,
                                      hipStream_t s);
hipError_t launch_load_accumulate(const int32_t *counts, int64_t n, int64_t *window, hipStream_t s);

}  // namespace craft
