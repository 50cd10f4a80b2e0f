// Grouped SwiGLU expert FFN over pre-packed weights (bf16, or E4M3 codes with a scale per
// row): the weight-streaming kernels.
//
// Under skewed routing a rank's slots split into a few with hundreds of rows and many with
// a handful, so the two grouped GEMMs of the expert FFN (Sec. 2.1) are partly matrix-bound
// and partly pure weight streaming: every weight byte of a live slot has to cross HBM once
// whatever the slot's row count.  What these kernels are built around:
//
//   * Expert weights are re-ordered once, outside the forward, into MFMA fragment order
//     (craft_pack_weights): for each group of output columns and each 32-wide step of the
//     contraction, the two 16 x 32 blocks that v_mfma_f32_16x16x32_bf16 consumes as its row
//     operand are stored as 64 lanes x 16 bytes each.  A wave reads its weights with fully
//     coalesced 1 KiB requests, straight into registers: no LDS, no transposition, and the
//     waves of a workgroup stream different column groups, so a workgroup requests no weight
//     byte twice.  For gate/up a group is the 16 gate rows of 16 output columns followed by
//     the 16 up rows of the same columns, which puts gate and up of one output into the same
//     lane and element of two accumulators: SwiGLU is applied in registers.
//   * The 16 x 16 x 32 shape, because the matrix pipelines' power sets the clock: on operands
//     like these a register-only loop of it sustains 2.05 PFLOP/s on this chip, one of
//     32 x 32 x 16 1.76-1.84.
//   * One workgroup of four waves per CU, one wave per SIMD, so a wave may use the whole
//     512-entry register file: a tile is up to 256 activation rows x 8 column groups, each
//     wave owning two groups x up to sixteen 16-row fragments (256 fp32 accumulators per
//     lane).  The large tile is what keeps the L2-to-CU traffic per flop low enough: a
//     weight fragment loaded into a CU is used against 256 rows, an activation fragment
//     against 128 (gate/up) or 256 (down) output columns.
//   * The weight stream runs 4 or 8 steps ahead of the MFMAs in a statically indexed register
//     ring; the activation rows (gathered through the dispatch permutation for gate/up) are
//     shared by the four waves through LDS: four stages of one 64-wide slab, filled two slabs
//     ahead by loads that write LDS directly (no registers, no LDS write instructions: those
//     hand over four data registers per lane, which the MFMAs' own operand fetches leave no
//     room for), one barrier per slab.  The contraction loop has no branch around a memory
//     operation, so the in-order load counter lets all of that stay in flight.
//   * Under full load a CU gets about 45 GB/s out of L2 whatever it asks for, and a 16-wide
//     piece of the contraction moves 8 KB of weights plus 1 KB per 32 rows into it: at
//     256 x 256 the tile needs those bytes about as fast as the MFMAs consume them, below that
//     it is bound by them.
//   * Weight fragments that a single tile reads (a cold slot's, a rider's, a busy slot's with
//     one row-tile) are requested with streaming loads, so that the L2 keeps the activation
//     rows and the weights that several tiles share.
//   * Row fragments beyond a tile's valid rows are skipped entirely (loads, LDS traffic,
//     MFMAs): a slot with 20 rows costs one eighth of the matrix work of a full tile while
//     streaming the same weights.
//   * Tiles are listed busiest slot first; in a launch of several rounds a slot's tiles come
//     as compact blocks of row-tiles x column tiles (ffn_common.h), so that the tiles running
//     at any time share activation rows and weight columns in the caches.  Each workgroup
//     takes one tile by position (the XCD-aware mapping of ffn_common.h, so neighbours in the
//     list start together on one XCD), then pulls further tiles from an atomic counter: the
//     cheap streaming tiles of the cold slots fill in behind the matrix-bound ones, or ride
//     along with them (see kRiderHostFrags in kernels.h).
#include "ffn_common.h"

namespace craft {
namespace {

// 32-wide weight steps kept in flight per column group.  Eight everywhere but in the tall tiles
// of the down GEMM: its contraction is short, and what a deeper ring requests before the first
// MFMA of a tile costs it more than the latency it covers (down GEMM at T = 32768: 438 -> 433 us).
// The row requests, which the compiler does not count, sit between the weight requests: its
// waits for a ring slot then wait for everything older as well, so a ring of eight steps covers
// about four steps of latency.
constexpr int ring_depth(int nxa, bool gateup) { return nxa >= 3 && !gateup ? 4 : 8; }
// The rider's weights always come from HBM (nobody else reads them): where the registers are
// there its ring runs twice as far ahead as the tile's own.
constexpr int rider_ring(int nxf, bool w8) { return w8 || nxf <= 4 ? 8 : 4; }
constexpr int NG = 2;             // column groups per wave in a full-width tile (1 in a half-width one)
constexpr int kPackGroups = 8;    // the packed stream is padded to whole full-width tiles
// An LDS stage holds one 64-wide slab of up to 256 activation rows, 128 bytes per row, no
// padding: the rows arrive by loads that write LDS directly, 64 lanes x 16 bytes to consecutive
// addresses.  So that the fragment reads (16 rows at one contraction offset) still spread over
// all banks (eight lanes, eight consecutive rows, are served per cycle), the eight 16-byte pieces
// of row r are stored in the order piece ^ (r & 7).
constexpr int XROWB = 64 * 2;
constexpr int XSTAGEB = kBM_packed * XROWB;
constexpr int kStages = 4;

typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
// A weight fragment as it sits in the ring: 8 bf16 values, or 8 E4M3 codes that are widened
// (exactly) right in front of the MFMAs that use them.
template <bool W8> struct WFrag { typedef bf16x8_t type; };
template <> struct WFrag<true> { typedef u32x2_t type; };

static __device__ __forceinline__ bf16x8_t widen(bf16x8_t w) { return w; }
static __device__ __forceinline__ bf16x8_t widen(u32x2_t w) {
    // two codes per conversion (bytes 0,1 / 2,3 of a word), then pairs of fp32 to bf16
    const f32x2_t a = __builtin_amdgcn_cvt_pk_f32_fp8(w[0], false), b = __builtin_amdgcn_cvt_pk_f32_fp8(w[0], true);
    const f32x2_t c = __builtin_amdgcn_cvt_pk_f32_fp8(w[1], false), d = __builtin_amdgcn_cvt_pk_f32_fp8(w[1], true);
    typedef unsigned int u32x4v __attribute__((ext_vector_type(4)));
    const u32x4v r = {bf16_pair(a[0], a[1]), bf16_pair(b[0], b[1]), bf16_pair(c[0], c[1]), bf16_pair(d[0], d[1])};
    return __builtin_bit_cast(bf16x8_t, r);
}
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));      // native vector: stays in VGPRs
template <bool W8> static __device__ __forceinline__ typename WFrag<W8>::type zero_fragment();
template <> __device__ __forceinline__ bf16x8_t zero_fragment<false>() {
    const u32x4_t z = {0u, 0u, 0u, 0u};
    return __builtin_bit_cast(bf16x8_t, z);
}
template <> __device__ __forceinline__ u32x2_t zero_fragment<true>() {
    const u32x2_t z = {0u, 0u};
    return z;
}
// Every global load of the contraction loop is addressed as a wave-uniform 64-bit base (scalar
// registers, advanced with scalar adds) plus a 32-bit byte offset per lane: no 64-bit vector
// arithmetic per request, and half the address registers to hand to the memory pipeline.
typedef const unsigned char *ubase_t;
static __device__ __forceinline__ ubase_t uniform_base(const void *p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<ubase_t>(((uint64_t)hi << 32) | lo);
}
// 16 bytes per lane from base + off straight into LDS at lds + 16 * lane (lds: the byte address
// of the wave's 1 KiB destination, wave-uniform; it goes through M0, which the compiler keeps
// nothing in across statements).  The compiler does not know that this is a load: it neither
// counts it among the outstanding requests (its own waits for other loads then only wait longer
// than needed, requests complete in order) nor waits for it before LDS reads (dma_wait does).
static __device__ __forceinline__ void dma_chunk(ubase_t base, uint32_t off, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds), "v"(off), "s"(base) : "memory");
}
// the same in two statements, with at least one instruction between them
static __device__ __forceinline__ void dma_to(uint32_t lds) { asm volatile("s_mov_b32 m0, %0" :: "s"(lds) : "memory"); }
static __device__ __forceinline__ void dma_request(ubase_t base, uint32_t off) {
    asm volatile("global_load_lds_dwordx4 %0, %1" :: "v"(off), "s"(base) : "memory");
}
// wait until at most N of this wave's requests are outstanding
template <int N> static __device__ __forceinline__ void dma_wait() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
// The lane's index inside its wave, counted afresh from the execution mask: with the wave's
// index kept in a scalar register no vector register has to carry the thread index through
// the contraction loops (it was spilled there, and its reload at the start of the epilogue
// waited for every request still in flight).
static __device__ __forceinline__ int lane_index() {
    int lane;                                      // volatile: counted where it is used, never kept
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane));
    return lane;
}
// A weight fragment that no other tile of the launch reads (a cold slot's: it has one
// row-tile): a streaming load, which leaves the L2 to the weights and rows that are shared.
template <bool ONCE, typename F>
static __device__ __forceinline__ F wload(ubase_t base, uint32_t &off) {
    // the lane's offset never changes inside a tile; widened to 64 bits once outside the loop it
    // would no longer be recognised as the 32-bit offset of a scalar-base request
    // (redefined in place, so that no copy is made)
    asm volatile("" : "+v"(off));
    const F __attribute__((address_space(1))) *p = (const F __attribute__((address_space(1))) *)(base + off);
    if (ONCE) return __builtin_nontemporal_load(p);
    return *p;
}

// Where a tile's operands come from.  The bases are wave-uniform; the weight offsets woff /
// wroff are the ring's next refill (the step that many ahead, held at the last step of the
// stream once it is reached) and move on by one step's worth of fragments per step.
struct Streams {
    ubase_t wb, wbr;           // packed weights of the tile's slot and of the rider's slot
    uint32_t wl, wlr;          // the lane's place in a step: (first fragment * 64 + lane) fragments, in bytes
    uint32_t woff, wroff;      // running refill offsets, in bytes
    uint32_t wstep, wlast;     // bytes per step; offset of the last step
    ubase_t xb, xbr;           // activation rows of the tile and of the rider
};

// acc += w x^T for a 16-row weight fragment and a 16-row activation fragment over 32
// contraction elements.  Written out as an instruction whose accumulator operand is both read
// and written (an accumulation register tuple, "+a"): a tall tile's 64 accumulators fill the
// accumulation half of the register file exactly, and every copy the register allocator makes
// when result and addend are two values costs moves through the other half.  The compiler does
// not know that this is a matrix instruction: the waits it would insert between a matrix
// instruction and a read of its result are the caller's (settle_accumulators) — inside the
// contraction loop an accumulator is touched again only a whole half-step later.
// FRESH: an operand has just been written by ordinary vector instructions (8-bit weights
// widened to bf16); a matrix instruction may read such a register two issue cycles later at
// the earliest, which the compiler would see to for an instruction it knows.
template <bool FRESH>
static __device__ __forceinline__ void mfma16(bf16x8_t w, bf16x8_t x, f32x4_t &c) {
    if (FRESH) asm("s_nop 1\n\tv_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(w), "v"(x));
    else asm("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(w), "v"(x));
}
// After the last matrix instruction and before the first ordinary read of an accumulator: more
// idle issue cycles than the longest wait the hardware asks for between the two.  Every
// accumulator then passes through an empty statement that is ordered behind the idle cycles
// (both are volatile), so that no read of it can be scheduled ahead of them.
template <int NGT, int NXF>
static __device__ __forceinline__ void settle_accumulators(f32x4_t (&acc)[NGT][2][2 * NXF], f32x4_t (&accr)[1][2][2],
                                                           bool rider) {
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
    for (int n = 0; n < NGT; ++n)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int g = 0; g < 2 * NXF; ++g) asm volatile("" : "+a"(acc[n][h][g]));
    if (rider)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 2; ++i) asm volatile("" : "+a"(accr[0][h][i]));
}

// Half of one 32-wide contraction step: the step's 2 NGT weight fragments (NGT column groups per
// wave, two 16-row fragments each) against the lower (HI = 0) or upper (HI = 1) NXF 16-row
// activation fragments of the tile, 2 NGT NXF MFMAs of 16 cycles.  A wave is alone on its SIMD,
// so whatever it issues between two MFMAs delays the second one unless it fits into the cycles
// the first one keeps the matrix pipeline busy: memory operations are therefore dealt out one
// per MFMA, and a scheduling barrier after each MFMA pins that order.
//   MFMA m < NXF           : + LDS read of fragment m of the FOLLOWING half-step into XN (this
//                            one runs on XC; a whole half-step of matrix work covers the latency)
//   the last MFMAs, STAGE  : a slab's first half-step requests the activation rows of the slab two
//   0                        ahead, which land in LDS by themselves (dma_chunk), one 32-row chunk
//                            behind each MFMA
//   HI, a fragment's last  : + refill of the ring slot that weight fragment came from
//   the rider, if any      : fragment NXF of the activations is 16 rows of a cold slot (its lower
//                            16 in the lower half-step) and meets one column group of that
//                            slot's weights (a ring of its own): two more MFMAs at the end
template <int NXF, int NGT, int R, int RR, int PW, int HI, int STAGE, bool W8, bool RIDER, bool ONCE>
__device__ __forceinline__ void packed_half(uint32_t xnext, Streams &sm,
                                            typename WFrag<W8>::type (&wq)[NGT][PW][2],
                                            typename WFrag<W8>::type (&wr)[RIDER ? rider_ring(NXF, W8) : 1][2],
                                            const bf16x8_t (&XC)[NXF + RIDER], bf16x8_t (&XN)[NXF + RIDER],
                                            f32x4_t (&acc)[NGT][2][2 * NXF], f32x4_t (&accr)[1][2][2], uint32_t dma_lds,
                                            const uint32_t (&xp)[NXF + RIDER], uint32_t koff) {
    typedef typename WFrag<W8>::type F;
    constexpr int NXA = NXF + (RIDER ? 1 : 0);     // activation fragments of a half in LDS, the rider's last
    constexpr int M = 2 * NGT * NXF + (RIDER ? 2 : 0);                 // MFMAs of this half-step
    constexpr int OP0 = M - 2 * NXA > 0 ? M - 2 * NXA : 0;             // MFMA behind which the first row chunk is prepared
    constexpr int NH = 1 - HI;                     // the half that is fetched from LDS meanwhile
    constexpr int RING_R = rider_ring(NXF, W8);
    if (HI) {
        sm.woff = min(sm.woff + sm.wstep, sm.wlast);
        if (RIDER) sm.wroff = min(sm.wroff + sm.wstep, sm.wlast);
    }
    const ubase_t wcur = sm.wb + sm.woff, wrcur = sm.wbr + sm.wroff;
    // xnext: the LDS address of the lane's piece of the first fragment to fetch.  Kept as one
    // register per half-step with the fragments at constant offsets from it: folded together
    // with the stage's offset the constants no longer fit the instruction and every read got an
    // address computation of its own.
    asm volatile("" : "+v"(xnext));
    typedef const bf16x8_t __attribute__((address_space(3))) *lds_frag_t;
    // what follows MFMA m
    auto after = [&](int m) __attribute__((always_inline)) {
        if (m < NXF) XN[m] = *(lds_frag_t)(uintptr_t)(xnext + 16 * (NH * NXF + m) * XROWB);
        if (RIDER && m == NXF) XN[NXA - 1] = *(lds_frag_t)(uintptr_t)(xnext + (32 * NXF + 16 * NH) * XROWB);
        if (STAGE == 0) {
#pragma unroll
            for (int i = 0; i < NXA; ++i) {
                // destination behind one MFMA, request behind the next: together they would
                // take longer to issue than an MFMA keeps the matrix pipeline busy
                if (m == (OP0 + 2 * i < M - 1 ? OP0 + 2 * i : M - 1)) dma_to(dma_lds + 32 * i * XROWB);
                if (m == (OP0 + 2 * i + 1 < M - 1 ? OP0 + 2 * i + 1 : M - 1)) dma_request(i < NXF ? sm.xb : sm.xbr, xp[i] + koff);
            }
        }
    };
#pragma unroll
    for (int n = 0; n < NGT; ++n) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const bf16x8_t wf = widen(wq[n][R][h]);
#pragma unroll
            for (int g = 0; g < NXF; ++g) {
                if (g == 0) mfma16<W8>(wf, XC[g], acc[n][h][HI * NXF + g]);
                else mfma16<false>(wf, XC[g], acc[n][h][HI * NXF + g]);
                after((2 * n + h) * NXF + g);
                if (HI && g == NXF - 1) wq[n][R][h] = wload<ONCE, F>(wcur + (2 * n + h) * 64 * (int)sizeof(F), sm.wl);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    if (RIDER) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            mfma16<W8>(widen(wr[RR % RING_R][h]), XC[NXA - 1], accr[0][h][HI]);
            after(2 * NGT * NXF + h);
            if (HI) wr[RR % RING_R][h] = wload<true, F>(wrcur + h * 64 * (int)sizeof(F), sm.wlr);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// One 64-wide slab U (0..3) of a group of four: two 32-wide steps, four half-steps.  The slab
// sits in LDS stage U (four stages: a group of four slabs goes once round them); X0 holds the
// lower fragments of its first step.  The first half-step requests the rows of slab U + 2 into
// stage (U + 2) % 4; before the barrier in front of the last half-step, which already reads the
// first fragments of slab U + 1, every wave waits for the requests it issued one slab ago (the
// rows of slab U + 1): since then it has issued the weight refills of three steps and the row
// requests of this slab, and requests complete in order.  A stage is overwritten two slabs after
// it was last read, with the barrier of the slab in between.
template <int NXF, int NGT, int U, int PW, bool W8, bool RIDER, bool ONCE>
__device__ __forceinline__ void packed_slab(int ks, int last_slab, int K, uint32_t kcb,
                                            uint32_t lds0, uint32_t lds_wave, uint32_t fo0,
                                            Streams &sm, const uint32_t (&xp)[NXF + RIDER],
                                            typename WFrag<W8>::type (&wq)[NGT][PW][2],
                                            typename WFrag<W8>::type (&wr)[RIDER ? rider_ring(NXF, W8) : 1][2],
                                            bf16x8_t (&X0)[NXF + RIDER],
                                            bf16x8_t (&X1)[NXF + RIDER], f32x4_t (&acc)[NGT][2][2 * NXF],
                                            f32x4_t (&accr)[1][2][2]) {
    constexpr int NXA = NXF + (RIDER ? 1 : 0);
    constexpr int V = 2 * NGT + (RIDER ? 2 : 0);   // weight requests per step
    // contraction offsets past the row are clamped into it: the weights there are zero
    // (in bytes, like the row offsets xp)
    const uint32_t koff = (uint32_t)min(min(ks + 2, last_slab) * 128 + (int)kcb, K * 2 - 16);
    const uint32_t dma_lds = lds_wave + (uint32_t)((U + 2) % kStages * XSTAGEB);
    const uint32_t cur = lds0 + U * XSTAGEB, nxt = lds0 + (U + 1) % kStages * XSTAGEB;
    const uint32_t fo1 = fo0 ^ 64u;                // the same fragment of the slab's second step
    packed_half<NXF, NGT, (U * 2 + 0) % PW, U * 2 + 0, PW, 0, 0, W8, RIDER, ONCE>(cur + fo0, sm, wq, wr, X0, X1, acc, accr, dma_lds, xp, koff);
    packed_half<NXF, NGT, (U * 2 + 0) % PW, U * 2 + 0, PW, 1, -1, W8, RIDER, ONCE>(cur + fo1, sm, wq, wr, X1, X0, acc, accr, dma_lds, xp, koff);
    packed_half<NXF, NGT, (U * 2 + 1) % PW, U * 2 + 1, PW, 0, -1, W8, RIDER, ONCE>(cur + fo1, sm, wq, wr, X0, X1, acc, accr, dma_lds, xp, koff);
    dma_wait<3 * V + NXA>();
    __syncthreads();
    packed_half<NXF, NGT, (U * 2 + 1) % PW, U * 2 + 1, PW, 1, -1, W8, RIDER, ONCE>(nxt + fo0, sm, wq, wr, X1, X0, acc, accr, dma_lds, xp, koff);
}

// Epilogue of 2 NF accumulator fragments of 16 rows x NGT column groups, which are the rows of
// tile t from its first on and the groups from group0 on.  Accumulator element v of lane l
// belongs to weight row 4 (l >> 4) + v of its 16-row weight fragment and activation row
// (l & 15) of its fragment: a lane holds 4 neighbouring output columns of one row, the lanes 16
// further on the next 4.  Two fragments at a time, neighbouring quarters of the wave trade
// pieces (v_permlane16_swap: the odd quarters of the first operand against the even quarters
// of the second), after which every lane owns 8 neighbouring columns of one of the two: 16-byte
// stores, half as many as 8-byte ones would be.  The two fragments are the two halves of a
// 32-column group (down), the same rows of two neighbouring 16-column groups (gate/up, after
// SwiGLU of the gate fragment with the up fragment of the same columns), or, where a wave has a
// single group, two fragments of rows.
template <bool GATEUP, int NGT, int NF, bool W8>
__device__ __forceinline__ void store_fragments(const FfnArgs &a, const Tile &t, const f32x4_t (&acc)[NGT][2][2 * NF],
                                                const float *wscale, int group0, int N, int32_t lo_pos) {
    constexpr int GC = GATEUP ? 16 : 32;
    // the lane's row and column offsets are derived here, after the contraction loop: shared
    // with values from before it they would sit in scratch through the loop, and every reload
    // would wait for the stores issued so far (loads and stores share one counter)
    const int lane = lane_index();
    unsigned short *outp = static_cast<unsigned short *>(GATEUP ? a.act : a.y);
    const int q = lane >> 4;
    // E4M3 weights: the fp32 scale of every weight row sits behind the stream (gate rows,
    // then up rows; or down rows) and multiplies the accumulator of that output column.
    // The scales depend on the column only: fetched once per group, not once per fragment.
    // sc[n][h]: gate/up h = 0 gate, 1 up (columns 16 (group0 + n) + 4 q ..); down h = half of the group
    float sc[NGT][2][4];
#pragma unroll
    for (int n = 0; n < NGT; ++n)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int c = 0; c < 4; ++c) sc[n][h][c] = 1.0f;
    if (W8) {
#pragma unroll
        for (int n = 0; n < NGT; ++n)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int c0 = min((group0 + n) * GC + (GATEUP ? 0 : 16 * h) + q * 4, N - 4);   // padding columns: any valid scale
                const float4 v = *reinterpret_cast<const float4 *>(wscale + (GATEUP ? h * N : 0) + c0);
                sc[n][h][0] = v.x; sc[n][h][1] = v.y; sc[n][h][2] = v.z; sc[n][h][3] = v.w;
            }
    }
    // the lane's 4 columns of fragment f, group n (down: half h of it), as two packed pairs
    auto piece = [&](int n, int h, int f, uint32_t (&p)[2]) __attribute__((always_inline)) {
        float v[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            v[c] = GATEUP ? silu_fast(acc[n][0][f][c] * sc[n][0][c]) * (acc[n][1][f][c] * sc[n][1][c])
                          : acc[n][h][f][c] * sc[n][h][c];
        p[0] = bf16_pair(v[0], v[1]);
        p[1] = bf16_pair(v[2], v[3]);
    };
    // x, y: the pieces of the first and second fragment of a pair; afterwards quarter q of the
    // wave holds columns 8 (q >> 1) .. + 7 of the first (q even) or second (q odd) fragment
    auto trade_and_store = [&](const uint32_t (&x)[2], const uint32_t (&y)[2], int m, int col) __attribute__((always_inline)) {
        const auto s0 = __builtin_amdgcn_permlane16_swap(x[0], y[0], false, false);
        const auto s1 = __builtin_amdgcn_permlane16_swap(x[1], y[1], false, false);
        if (m < t.rows && col < N) {
            u32x4_t v;
            v[0] = s0[0]; v[1] = s1[0]; v[2] = s0[1]; v[3] = s1[1];
            unsigned short *orow = outp + (int64_t)(t.pos0 + t.m0 + m - lo_pos) * N;
            *reinterpret_cast<u32x4_t *>(orow + col) = v;
        }
    };
    // Fragment by fragment, all column groups of the wave before the next fragment: the stores
    // that fill one 128-byte line of an output row (a wave's 64 columns of the down GEMM) follow
    // one another, so the line leaves the L2 whole instead of in pieces.
    if (!GATEUP) {
#pragma unroll
        for (int f = 0; f < 2 * NF; ++f)
#pragma unroll
            for (int n = 0; n < NGT; ++n) {
                uint32_t x[2], y[2];
                piece(n, 0, f, x);
                piece(n, 1, f, y);
                trade_and_store(x, y, f * 16 + (lane & 15), (group0 + n) * GC + (q & 1) * 16 + (q >> 1) * 8);
            }
    } else if (NGT == 2) {
#pragma unroll
        for (int f = 0; f < 2 * NF; ++f) {
            uint32_t x[2], y[2];
            piece(0, 0, f, x);
            piece(NGT - 1, 0, f, y);
            trade_and_store(x, y, f * 16 + (lane & 15), (group0 + (q & 1)) * GC + (q >> 1) * 8);
        }
    } else {
#pragma unroll
        for (int f = 0; f < 2 * NF; f += 2) {
            uint32_t x[2], y[2];
            piece(0, 0, f, x);
            piece(0, 0, f + 1, y);
            trade_and_store(x, y, (f + (q & 1)) * 16 + (lane & 15), group0 * GC + (q >> 1) * 8);
        }
    }
}

// One tile with NXF live 32-row activation fragments of its own slot (2 NXF fragments of 16
// rows: NXF lower, NXF upper) and, with RIDER, one more 32-row fragment of a cold slot (tile r:
// up to 32 rows, half a column tile starting at r.n0) that meets one column group of that
// slot's weights per wave.
template <bool GATEUP, int NXF, int NGT, bool W8, bool RIDER, bool ONCE>
__device__ __forceinline__ int32_t packed_tile(const FfnArgs &a, const Tile &t, const Tile &r, unsigned char *smem,
                                               int K, int N, int ngroups, int nk4, int32_t lo_pos, int32_t *counter,
                                               int wave_id) {
    constexpr int GC = GATEUP ? 16 : 32;
    constexpr int NXA = NXF + (RIDER ? 1 : 0);
    constexpr int PW = ring_depth(NXA, GATEUP);
    constexpr int RING_R = rider_ring(NXF, W8);
    // The lane's constants (LDS offsets and the like) are derived afresh in every tile: hoisted
    // out of the tile loop they would stay live through the tallest tile, which has no
    // register to spare, and come back from scratch inside every contraction loop.
    const int lane = lane_index(), wave = wave_id;
    const int tid = wave * 64 + lane;
    const int lr = tid >> 3;
    // the lane's part in fetching a 32-row chunk: row lr of it, and the 16-byte piece of the slab
    // that belongs at place (lane & 7) of that row in LDS
    const uint32_t kcb = (uint32_t)(((lane & 7) ^ (lr & 7)) * 16);
    // the lane's fragment reads: row (lane & 15) of a 16-row fragment, piece (lane >> 4) of the
    // slab's first step where that row keeps it
    const uint32_t fo0 = (uint32_t)((lane & 15) * XROWB + (((lane >> 4) ^ (lane & 7)) & 7) * 16);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const uint32_t lds_wave = lds0 + (uint32_t)__builtin_amdgcn_readfirstlane(wave * 8 * XROWB);
    const int ksteps = nk4 * 8;                    // 32-wide steps
    const int group0 = t.n0 / GC + wave * NGT;     // this wave's first column group
    const int group_r = r.n0 / GC + wave;          // and its one group of the rider
    const void *wbase = GATEUP ? a.wp_gateup[t.slot] : a.wp_down[t.slot];
    const void *wbase_r = RIDER ? (GATEUP ? a.wp_gateup[r.slot] : a.wp_down[r.slot]) : wbase;
    // step-major stream: the fragments of all column groups for one step are adjacent, two per
    // group.  The packed buffer holds a multiple of kPackGroups groups (zero padded), so every
    // wave of a tile has a stream to read even past the last real column.
    const int groups_padded = (ngroups + kPackGroups - 1) / kPackGroups * kPackGroups;
    typedef typename WFrag<W8>::type F;
    Streams sm;
    sm.wb = uniform_base(wbase);
    sm.wbr = uniform_base(wbase_r);
    sm.wl = (uint32_t)(group0 * 128 + lane) * (uint32_t)sizeof(F);
    sm.wlr = (uint32_t)(group_r * 128 + lane) * (uint32_t)sizeof(F);
    sm.wstep = (uint32_t)groups_padded * 128u * (uint32_t)sizeof(F);
    sm.wlast = (uint32_t)(ksteps - 1) * sm.wstep;  // the host checks that a packed matrix stays below 4 GiB
    sm.woff = (uint32_t)(PW - 1) * sm.wstep;       // the loop's first refill is step PW (ksteps >= 8 >= PW)
    sm.wroff = (uint32_t)(RING_R - 1) * sm.wstep;
    // Activation rows as 32-bit byte offsets from a uniform base.  Gate/up gathers token rows
    // from all over x (the host checks that x stays below 4 GiB); the down GEMM's rows follow
    // one another from the tile's first row on, the rider's from the rider's first row.
    const uint32_t row_bytes = (uint32_t)K * 2u;
    if (GATEUP) {
        sm.xb = sm.xbr = static_cast<ubase_t>(a.x);
    } else {
        const int32_t row0 = __builtin_amdgcn_readfirstlane(t.pos0 + t.m0 - lo_pos);
        const int32_t row0r = __builtin_amdgcn_readfirstlane(r.pos0 + r.m0 - lo_pos);
        sm.xb = static_cast<ubase_t>(a.act) + (int64_t)row0 * row_bytes;
        sm.xbr = static_cast<ubase_t>(a.act) + (int64_t)row0r * row_bytes;
    }
    uint32_t xp[NXA];
#pragma unroll
    for (int i = 0; i < NXA; ++i) {
        const bool own = i < NXF;
        const int rr = own ? min(lr + 32 * i, t.rows - 1) : min(lr, r.rows - 1);
        const int32_t pos = own ? t.pos0 + t.m0 + rr : r.pos0 + r.m0 + rr;
        xp[i] = (uint32_t)(GATEUP ? a.src[pos] / a.k : rr) * row_bytes;
    }

    f32x4_t acc[NGT][2][2 * NXF], accr[1][2][2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 2; ++i) accr[0][h][i] = (f32x4_t)(0.0f);
#pragma unroll
    for (int n = 0; n < NGT; ++n)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int g = 0; g < 2 * NXF; ++g) acc[n][h][g] = (f32x4_t)(0.0f);

    // Request order: half the weight rings, the first two activation slabs (into stages 0 and
    // 1), the other half of the rings.  The first slab is complete once at most the requests
    // issued after it are outstanding; the second is waited for in the first slab of the loop,
    // which finds at least as many younger requests as any later slab does.
    F wq[NGT][PW][2], wr[RIDER ? RING_R : 1][2];
    {
#pragma unroll
        for (int j = 0; j < PW / 2; ++j)
#pragma unroll
            for (int n = 0; n < NGT; ++n)
#pragma unroll
                for (int h = 0; h < 2; ++h) wq[n][j][h] = wload<ONCE, F>(sm.wb + (uint32_t)j * sm.wstep + (2 * n + h) * 64 * (int)sizeof(F), sm.wl);
        if (RIDER)
#pragma unroll
            for (int j = 0; j < RING_R / 2; ++j)
#pragma unroll
                for (int h = 0; h < 2; ++h) wr[j][h] = wload<true, F>(sm.wbr + (uint32_t)j * sm.wstep + h * 64 * (int)sizeof(F), sm.wlr);
        if (!RIDER) wr[0][0] = wr[0][1] = zero_fragment<W8>();    // placeholders that no MFMA reads
        const uint32_t k0 = (uint32_t)min((int)kcb, K * 2 - 16), k1 = (uint32_t)min(128 + (int)kcb, K * 2 - 16);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NXA; ++i) dma_chunk(i < NXF ? sm.xb : sm.xbr, xp[i] + k0, lds_wave + 32 * i * XROWB);
#pragma unroll
        for (int i = 0; i < NXA; ++i) dma_chunk(i < NXF ? sm.xb : sm.xbr, xp[i] + k1, lds_wave + XSTAGEB + 32 * i * XROWB);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = PW / 2; j < PW; ++j)
#pragma unroll
            for (int n = 0; n < NGT; ++n)
#pragma unroll
                for (int h = 0; h < 2; ++h) wq[n][j][h] = wload<ONCE, F>(sm.wb + (uint32_t)j * sm.wstep + (2 * n + h) * 64 * (int)sizeof(F), sm.wl);
        if (RIDER)
#pragma unroll
            for (int j = RING_R / 2; j < RING_R; ++j)
#pragma unroll
                for (int h = 0; h < 2; ++h) wr[j][h] = wload<true, F>(sm.wbr + (uint32_t)j * sm.wstep + h * 64 * (int)sizeof(F), sm.wlr);
        __builtin_amdgcn_sched_barrier(0);
        dma_wait<NXA + (PW - PW / 2) * 2 * NGT + (RIDER ? (RING_R - RING_R / 2) * 2 : 0)>();
    }
    __syncthreads();

    // the lower fragments of the first step (the rider's 32 rows sit behind the tile's own)
    bf16x8_t x0[NXA], x1[NXA];
#pragma unroll
    for (int g = 0; g < NXF; ++g) x0[g] = *reinterpret_cast<const bf16x8_t *>(smem + fo0 + g * 16 * XROWB);
    if (RIDER) x0[NXA - 1] = *reinterpret_cast<const bf16x8_t *>(smem + fo0 + 32 * NXF * XROWB);

    const int last_slab = nk4 * 4 - 1;
    for (int ks = 0; ks <= last_slab; ks += 4) {
        packed_slab<NXF, NGT, 0, PW, W8, RIDER, ONCE>(ks + 0, last_slab, K, kcb, lds0, lds_wave, fo0, sm, xp, wq, wr, x0, x1, acc, accr);
        packed_slab<NXF, NGT, 1, PW, W8, RIDER, ONCE>(ks + 1, last_slab, K, kcb, lds0, lds_wave, fo0, sm, xp, wq, wr, x0, x1, acc, accr);
        packed_slab<NXF, NGT, 2, PW, W8, RIDER, ONCE>(ks + 2, last_slab, K, kcb, lds0, lds_wave, fo0, sm, xp, wq, wr, x0, x1, acc, accr);
        packed_slab<NXF, NGT, 3, PW, W8, RIDER, ONCE>(ks + 3, last_slab, K, kcb, lds0, lds_wave, fo0, sm, xp, wq, wr, x0, x1, acc, accr);
    }
    // the last slabs have requested rows past the end of the contraction (the last slab again):
    // nothing may still be on its way into LDS when the tile, and perhaps the workgroup, ends
    dma_wait<0>();

    // The next work item is claimed before the epilogue and looked at after it: the counter's
    // round trip runs while the results are converted and stored.
    // (an increment rather than an add: the compiler rewrites an add of a uniform value into a
    // wave-wide reduction whose result it waits for on the spot)
    int32_t claimed = 0;
    if (tid == 0) claimed = (int32_t)atomicInc(reinterpret_cast<unsigned int *>(counter), 0xffffffffu);
    settle_accumulators<NGT, NXF>(acc, accr, RIDER);
    const size_t scale_off = (size_t)groups_padded * ksteps * 1024;   // E4M3: row scales behind the codes
    store_fragments<GATEUP, NGT, NXF, W8>(
        a, t, acc, reinterpret_cast<const float *>(static_cast<const unsigned char *>(wbase) + scale_off),
        group0, N, lo_pos);
    if (RIDER)   // the rider's accumulators are those of a one-fragment, one-group tile
        store_fragments<GATEUP, 1, 1, W8>(
            a, r, accr, reinterpret_cast<const float *>(static_cast<const unsigned char *>(wbase_r) + scale_off),
            group_r, N, lo_pos);
    return claimed;
}

// a busy slot's tile of F fragments, with or without a rider; the weights of a slot with a single
// row-tile are read by this tile alone and streamed
#define HOT(F, RIDE)                                                                                   \
    do {                                                                                               \
        if (t.single) claimed = packed_tile<GATEUP, F, NG, W8, RIDE, true>(a, t, r, smem, K, N, ngroups, nk4, lo_pos, counter, wave_id);   \
        else claimed = packed_tile<GATEUP, F, NG, W8, RIDE, false>(a, t, r, smem, K, N, ngroups, nk4, lo_pos, counter, wave_id);           \
    } while (0)

template <bool GATEUP, bool W8>
__global__ __launch_bounds__(256, 1) void ffn_packed_kernel(FfnArgs a) {
    __shared__ __attribute__((aligned(16))) unsigned char smem[kStages * XSTAGEB];
    __shared__ int64_t next_item;
    __shared__ TileTables tt;
    const int wave_id = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int32_t *mt_start = a.mt_start + (GATEUP ? 0 : a.nslots + 1);
    const bool small = a.nslots <= TileTables::kMaxSlots;
    if (small) load_tile_tables(a, mt_start, tt);
    const int K = GATEUP ? a.H : a.I;
    const int N = GATEUP ? a.I : a.H;
    constexpr int GC = GATEUP ? 16 : 32;           // output columns per weight group
    constexpr int BN = 4 * NG * GC;                // output columns per tile
    const int ngroups = (N + GC - 1) / GC;
    const int nt = (N + BN - 1) / BN;
    const int nk4 = (K + 255) / 256;               // groups of four 64-wide slabs
    // The tile list: the busy slots' tiles (row-tiles x nt column tiles each, found through
    // mt_start), the first `carried` of them with a rider unit each, then what is left of the
    // cold slots' units as tiles of their own (one row-tile, 2 nt half-width column tiles per
    // slot).  Units are counted over the cold slots in list order: a two-fragment slot has
    // 4 nt (fragment-major), a one-fragment slot 2 nt.
    const int32_t hot = a.ctrl[CTRL_HOT_SLOTS], live = a.ctrl[CTRL_LIVE_SLOTS];
    const int32_t cold2 = a.ctrl[CTRL_COLD2_SLOTS];
    const int64_t carried = a.ctrl[GATEUP ? CTRL_RIDERS_GATEUP : CTRL_RIDERS_DOWN];
    const int64_t units2 = (int64_t)cold2 * 4 * nt;
    const int64_t hot_tiles = (int64_t)mt_start[hot] * nt;
    const int64_t cold_tiles = carried <= units2 ? (int64_t)(live - hot) * 2 * nt - carried / 2
                                                 : (int64_t)(live - hot - cold2) * 2 * nt - (carried - units2);
    const int64_t total = hot_tiles + cold_tiles;
    const int32_t lo_pos = a.slot_off[a.s_lo];
    const int32_t fmax = GATEUP ? a.frags_gu : a.frags_dn;
    // A launch of more than two rounds of busy tiles lists a slot's tiles block by block
    // (ffn_common.h); a shorter one column by column, which packs its end best.
    int32_t *const counter = a.ctrl + (GATEUP ? CTRL_WORK_GATEUP : CTRL_WORK_DOWN);
    const bool blocked = hot_tiles > 2 * (int64_t)gridDim.x;
    // whole slot at position pos of the busiest-first order, as a tile
    auto slot_tile = [&](int32_t pos) {
        Tile t;
        t.slot = small ? tt.order[pos] : a.order[pos];
        t.pos0 = small ? tt.slot_off[t.slot] : a.slot_off[a.s_lo + t.slot];
        t.rows = (small ? tt.slot_off[t.slot + 1] : a.slot_off[a.s_lo + t.slot + 1]) - t.pos0;
        t.m0 = 0;
        t.n0 = 0;
        t.mtile = 0;
        t.single = 1;
        return t;
    };

    int64_t w = xcd_major_id();                    // first tile by position, the rest on demand
    while (w < total) {
        int32_t claimed = 0;                       // thread 0: the counter's answer, fetched inside the tile
        if (w < hot_tiles) {
            const Tile t = small ? decode_tile(a, tt, w, nt, BN, fmax, blocked)
                                 : decode_tile(a, mt_start, w, nt, BN, fmax, blocked);
            const int frags = (t.rows + 31) >> 5;  // live 32-row fragments of this tile
            Tile r = t;
            bool ride = w < carried && frags <= kRiderHostFrags;
            if (ride) {                            // unit w: which cold slot, fragment and half column tile
                const int64_t v = w < units2 ? w : w - units2;
                r = slot_tile(hot + (int32_t)(w < units2 ? v / (4 * nt) : cold2 + v / (2 * nt)));
                r.m0 = w < units2 ? (int32_t)(v % (4 * nt) / (2 * nt)) * 32 : 0;
                r.rows = min(32, r.rows - r.m0);
                r.n0 = (int32_t)(v % (2 * nt)) * (BN / 2);
                ride = r.n0 < N;                   // the last half may lie past the matrix
            }
            if (ride) {
                switch (frags) {
                    case 1: HOT(1, true); break;
                    case 2: HOT(2, true); break;
                    case 3: HOT(3, true); break;
                    case 4: HOT(4, true); break;
                    case 5: HOT(5, true); break;
                    case 6: HOT(6, true); break;
                    default: HOT(7, true); break;
                }
            } else {
                switch (frags) {
                    case 1: HOT(1, false); break;
                    case 2: HOT(2, false); break;
                    case 3: HOT(3, false); break;
                    case 4: HOT(4, false); break;
                    case 5: HOT(5, false); break;
                    case 6: HOT(6, false); break;
                    case 7: HOT(7, false); break;
                    default: HOT(8, false); break;
                }
            }
        } else {
            // what the riders left: whole slots (both fragments in one tile) while inside the
            // two-fragment slots, single units after them
            const int64_t cw = w - hot_tiles;
            const int64_t v = carried <= units2 ? cw : cw + (carried - units2);
            const int32_t c = carried <= units2 ? (int32_t)(carried / (4 * nt) + v / (2 * nt))
                                                : cold2 + (int32_t)(v / (2 * nt));
            Tile t = slot_tile(hot + c);
            t.n0 = (int32_t)(v % (2 * nt)) * (BN / 2);
            if (t.n0 < N) {                        // the last half may lie past the matrix
                if (t.rows <= 32) claimed = packed_tile<GATEUP, 1, 1, W8, false, true>(a, t, t, smem, K, N, ngroups, nk4, lo_pos, counter, wave_id);
                else claimed = packed_tile<GATEUP, 2, 1, W8, false, true>(a, t, t, smem, K, N, ngroups, nk4, lo_pos, counter, wave_id);
            } else if (wave_id == 0 && lane_index() == 0) {
                claimed = (int32_t)atomicInc(reinterpret_cast<unsigned int *>(counter), 0xffffffffu);
            }
        }
        if (wave_id == 0 && lane_index() == 0) next_item = (int64_t)gridDim.x + claimed;
        __syncthreads();
        w = next_item;
        __syncthreads();
    }
}

// One 16-byte chunk of the packed stream per thread: chunk ((step * groups + group) * 2 + half) * 64 + lane.
//   gate/up : group g = output columns 16g..16g+15; half 0 = gate rows 16g..16g+15, half 1 = the
//             up rows of the same columns
//   down    : group g = output columns 32g..32g+31; half h = down rows 32g+16h..+15
// Lane l of 32-wide step s holds row (l & 15) of its half, contraction elements 32s + 8(l>>4) .. +7:
// the row operand of one v_mfma_f32_16x16x32_bf16.  Rows and contraction elements past the matrix are zero.
__global__ void pack_kernel(const unsigned short *wa, const unsigned short *wb, int rows, int K,
                            int gc, int64_t nchunks, int ksteps, uint4 *out) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= nchunks) return;
    const int l = (int)(c & 63);
    const int h = (int)(c >> 6) & 1;
    const int64_t sg = c >> 7;                   // step-major
    const int64_t ngroups = nchunks / 128 / ksteps;   // padded to whole tiles of 8 groups
    const int s = (int)(sg / ngroups);
    const int64_t g = sg % ngroups;
    const int r = l & 15;
    const int k0 = 32 * s + 8 * (l >> 4);
    int64_t row;
    const unsigned short *src;
    if (gc == 16) { row = g * 16 + r; src = h ? wb : wa; }
    else { row = g * 32 + 16 * h + r; src = wa; }
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < rows && k0 < K) v = *reinterpret_cast<const uint4 *>(src + row * K + k0);
    out[c] = v;
}

template <bool GATEUP>
hipError_t launch_packed(const FfnArgs &a, hipStream_t s) {
    if (a.nslots <= 0 || a.max_rows <= 0) return hipSuccess;
    const int N = GATEUP ? a.I : a.H;
    const int bn = GATEUP ? 128 : 256;
    const int64_t nt = (N + bn - 1) / bn;
    const int64_t bound = (a.max_rows / (32 * std::abs(GATEUP ? a.frags_gu : a.frags_dn)) + 2 * a.nslots) * nt;
    int64_t grid = std::min<int64_t>(bound, (int64_t)a.num_cu);
    grid = std::max<int64_t>(8, (grid + 7) / 8 * 8);
    if (a.w8) hipLaunchKernelGGL((ffn_packed_kernel<GATEUP, true>), dim3((unsigned)grid), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((ffn_packed_kernel<GATEUP, false>), dim3((unsigned)grid), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gateup_packed(const FfnArgs &a, hipStream_t s) { return launch_packed<true>(a, s); }
hipError_t launch_down_packed(const FfnArgs &a, hipStream_t s) { return launch_packed<false>(a, s); }

void packed_sizes(int32_t H, int32_t I, size_t *gateup_bytes, size_t *down_bytes) {
    const size_t gu_groups = ((size_t)(I + 15) / 16 + 7) / 8 * 8, gu_steps = (size_t)(H + 255) / 256 * 16;
    const size_t dn_groups = ((size_t)(H + 31) / 32 + 7) / 8 * 8, dn_steps = (size_t)(I + 255) / 256 * 16;
    *gateup_bytes = gu_groups * gu_steps * 1024;
    *down_bytes = dn_groups * dn_steps * 1024;
}

hipError_t launch_pack(int32_t H, int32_t I, const void *wg, const void *wu, const void *wd,
                       void *pgu, void *pdn, hipStream_t s) {
    size_t gub, dnb;
    packed_sizes(H, I, &gub, &dnb);
    const int64_t c1 = (int64_t)(gub / 16), c2 = (int64_t)(dnb / 16);
    hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((c1 + 255) / 256)), dim3(256), 0, s,
                       static_cast<const unsigned short *>(wg), static_cast<const unsigned short *>(wu),
                       I, H, 16, c1, (H + 255) / 256 * 8, static_cast<uint4 *>(pgu));
    hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((c2 + 255) / 256)), dim3(256), 0, s,
                       static_cast<const unsigned short *>(wd), static_cast<const unsigned short *>(wd),
                       H, I, 32, c2, (I + 255) / 256 * 8, static_cast<uint4 *>(pdn));
    return hipGetLastError();
}

}  // namespace craft
