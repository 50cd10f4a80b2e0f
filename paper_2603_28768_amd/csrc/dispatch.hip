// Expert-load counts and replica-aware stable dispatch (Sec. 1 / Alg. 1: a replicated
// expert's tokens are spread evenly over its copies).
//
// The i-th assignment (in flat token-major order) that names expert e goes to that
// expert's copy i mod c_e, and is the (i div c_e)-th row of that copy's slot.  i is
// assembled from two parts: the assignment's rank inside its 32-token block (recorded by
// the routing kernel) and the number of assignments to e in all earlier blocks, which
// scan_kernel produces as an exclusive prefix over blocks.  No result depends on the
// order in which atomics retire, so indices are reproducible bit for bit.
#include "kernels.h"

namespace craft {
namespace {

constexpr int kScanThreads = 1024;
constexpr int kScanWaves = kScanThreads / 64;
static_assert(kScanChunk % kScanWaves == 0, "a chunk is dealt to the waves in equal parts");

// Exclusive scan over the workgroup of one value per thread (wave shuffles, then one LDS
// exchange between the WAVES waves).  Returns the exclusive prefix; *total gets the sum.
template <int WAVES>
__device__ __forceinline__ int32_t block_exclusive_scan(int32_t v, int32_t *wsum /*[WAVES]*/,
                                                        int32_t *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int32_t o = __shfl_up(inc, off, 64);
        if (lane >= off) inc += o;
    }
    __syncthreads();                       // wsum may still be read from an earlier scan
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    int32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
        const int32_t s = wsum[w];
        if (w < wave) before += s;
        all += s;
    }
    *total = all;
    return before + inc - v;
}

// Blocks of tokens are taken in chunks of kScanChunk; a workgroup handles one chunk for 64
// experts (a single workgroup walks over all experts when there is only one chunk).  Wave w
// owns 16 consecutive blocks of the chunk and a lane owns one expert: each wave sums its
// blocks (kept in registers), the waves' sums are prefix-combined through LDS, and the
// per-block counts are rewritten as exclusive prefixes inside the chunk.  With several
// chunks the chunk totals go to memory and the workgroup that finishes last (ticket
// counter) turns them into per-chunk bases, which the dispatch kernel adds.  That workgroup
// (trivially the only one) also derives what needs all counts and what the dispatch indices
// wait for: rows per slot, slot offsets and the rank's row count.
__global__ __launch_bounds__(kScanThreads) void scan_kernel(ScanArgs a) {
    __shared__ int32_t part[kScanWaves][64];
    __shared__ int32_t wsum[kScanWaves];
    __shared__ int32_t cnt_lds[1024];
    __shared__ int32_t last_flag;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int kKeep = kScanChunk / kScanWaves;         // blocks per wave
    const bool single = gridDim.x == 1;
    const int groups = (a.E + 63) / 64;
    const int chunk = single ? 0 : (int)blockIdx.x / groups;
    const int cb1 = min(a.NB, (chunk + 1) * kScanChunk);
    const int b0 = min(cb1, chunk * kScanChunk + wave * kKeep), b1 = min(cb1, b0 + kKeep);

    for (int grp = single ? 0 : (int)blockIdx.x % groups; grp < (single ? groups : (int)blockIdx.x % groups + 1); ++grp) {
        const int e = grp * 64 + lane;
        int32_t keep[kKeep];
        int32_t sum = 0;
        if (e < a.E) {
#pragma unroll
            for (int i = 0; i < kKeep; ++i) {
                keep[i] = b0 + i < b1 ? a.hist[(int64_t)(b0 + i) * a.E + e] : 0;
                sum += keep[i];
            }
        }
        part[wave][lane] = sum;
        __syncthreads();
        int32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kScanWaves; ++w) {
            const int32_t v = part[w][lane];
            if (w < wave) before += v;
            total += v;
        }
        if (e < a.E) {
            int32_t run = before;
#pragma unroll
            for (int i = 0; i < kKeep; ++i)
                if (b0 + i < b1) { a.hist[(int64_t)(b0 + i) * a.E + e] = run; run += keep[i]; }
            if (wave == 0) {
                if (single) {
                    a.counts[e] = total;
                    if (a.user_counts) a.user_counts[e] = total;
                    cnt_lds[e] = total;
                } else {
                    a.chunk_tot[(int64_t)chunk * a.E + e] = total;
                }
            }
        }
        __syncthreads();                   // `part` is reused by the next group
    }

    if (!single) {
        // publish, then take a ticket
        __threadfence();
        __syncthreads();
        if (threadIdx.x == 0) {
            const int32_t ticket = atomicAdd(&a.ctrl[CTRL_TICKET], 1);
            last_flag = ticket == (int32_t)gridDim.x - 1;
        }
        __syncthreads();
        if (!last_flag) return;
        __threadfence();
        // chunk totals -> chunk bases and the experts' counts
        const int chunks = (int)gridDim.x / groups;
        for (int32_t e = threadIdx.x; e < a.E; e += kScanThreads) {
            int32_t run = 0;
            for (int c = 0; c < chunks; ++c) {
                a.chunk_base[(int64_t)c * a.E + e] = run;
                run += __hip_atomic_load(a.chunk_tot + (int64_t)c * a.E + e, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
            }
            a.counts[e] = run;
            if (a.user_counts) a.user_counts[e] = run;
            cnt_lds[e] = run;
        }
    }
    __syncthreads();

    const craft_tables_header *hdr = reinterpret_cast<const craft_tables_header *>(a.tables);
    const int32_t *copies = a.tables + hdr->off_copies;
    const int32_t *slot_expert = a.tables + hdr->off_slot_expert;
    const int32_t *slot_copy = a.tables + hdr->off_slot_copy;

    // rows of slot p: tokens i < n of its expert with i mod c == q.  Slots are taken in
    // chunks of one per thread; `carry` is the running offset across chunks.
    // The two offsets that bound the rank's rows stay in LDS: reading them back from global
    // memory would be one more dependent round trip in this serial tail.
    __shared__ int32_t bound_pos[2];
    int32_t carry = 0, lo_pos = 0, hi_pos = 0;
    for (int32_t base = 0; base < a.S; base += kScanThreads) {
        const int32_t p = base + threadIdx.x;
        int32_t r = 0;
        if (p < a.S) {
            const int32_t ex = slot_expert[p];
            const int32_t n = cnt_lds[ex], c = copies[ex], q = slot_copy[p];
            r = n > q ? (n - q + c - 1) / c : 0;
        }
        int32_t chunk_total;
        const int32_t off = carry + block_exclusive_scan<kScanWaves>(r, wsum, &chunk_total);
        if (p < a.S) {
            a.slot_cnt[p] = r;
            a.slot_off[p] = off;
            if (a.user_slot_cnt) a.user_slot_cnt[p] = r;
            if (a.user_slot_off) a.user_slot_off[p] = off;
            if (p == a.s_lo) bound_pos[0] = off;
            if (p == a.s_hi) bound_pos[1] = off;
        }
        carry += chunk_total;
    }
    if (threadIdx.x == 0) {
        a.slot_off[a.S] = carry;
        if (a.user_slot_off) a.user_slot_off[a.S] = carry;
    }
    __syncthreads();
    lo_pos = a.s_lo < a.S ? bound_pos[0] : carry;
    hi_pos = a.s_hi < a.S ? bound_pos[1] : carry;
    // this rank's rows; refuse the batch when they exceed the staging buffers
    const int32_t rank_rows = hi_pos - lo_pos;
    const bool ovf = (int64_t)rank_rows > a.max_rows;
    if (threadIdx.x == 0) {
        a.ctrl[CTRL_ROWS] = rank_rows;
        a.ctrl[CTRL_OVERFLOW] = ovf ? 1 : 0;
        a.ctrl[CTRL_TICKET] = 0;
    }
}

// What the grouped GEMMs need beyond the slot offsets: the rank's slots ordered by rows, the
// row-tile prefixes of both GEMMs over that order and the rider units.  None of it is needed
// for the dispatch indices, so it is built by one extra workgroup of the dispatch launch
// while the others write dest / src, instead of at the end of the scan's serial tail.
constexpr int kTableThreads = 256;
__device__ void build_tile_tables(const DispatchArgs &a) {
    __shared__ int32_t rank_slot_rows[1024];
    __shared__ int32_t sorted_rows[1024];
    __shared__ int32_t wsum[kTableThreads / 64];
    __shared__ int32_t prefix_len[3];
    __shared__ int32_t hot_mtiles;
    const int32_t nslots = a.s_hi - a.s_lo;
    const bool ovf = a.ctrl[CTRL_OVERFLOW] != 0;
    for (int32_t sl = threadIdx.x; sl < nslots; sl += kTableThreads) rank_slot_rows[sl] = a.slot_cnt[a.s_lo + sl];
    if (threadIdx.x < 3) prefix_len[threadIdx.x] = 0;
    __syncthreads();
    // Order the rank's slots by rows, busiest first (ties: lower slot), so the tile list
    // starts with the matrix-bound tiles and ends with the cheap weight-streaming ones.
    for (int32_t sl = threadIdx.x; sl < nslots; sl += kTableThreads) {
        const int32_t mine = rank_slot_rows[sl];
        int32_t pos = 0;
        for (int32_t j = 0; j < nslots; ++j) {
            const int32_t other = rank_slot_rows[j];
            pos += (other > mine || (other == mine && j < sl)) ? 1 : 0;
        }
        a.order[pos] = sl;
        sorted_rows[pos] = mine;
    }
    __syncthreads();
    // the busy and the live slots are prefixes of the busiest-first order, and so are the slots
    // with more than one fragment
    for (int32_t pos = threadIdx.x; pos < nslots; pos += kTableThreads) {
        const int32_t r = sorted_rows[pos], nxt = pos + 1 < nslots ? sorted_rows[pos + 1] : 0;
        if (r > kColdRows && nxt <= kColdRows) prefix_len[0] = pos + 1;
        if (r > 0 && nxt <= 0) prefix_len[1] = pos + 1;
        if (r > 32 && nxt <= 32) prefix_len[2] = pos + 1;
    }
    __syncthreads();
    const int32_t hot = ovf ? 0 : prefix_len[0], live = ovf ? 0 : prefix_len[1];
    const int32_t ncold = live - hot;
    const int32_t ncold2 = max(0, min(prefix_len[2], live) - hot);   // cold slots with two fragments
    // row-tiles per slot: its 32-row fragments over the launch's tile height, rounded up
    int32_t mtotal[2], riders[2];
    for (int kind = 0; kind < 2; ++kind) {
        const int32_t fmax = abs(kind == 0 ? a.frags_gu : a.frags_dn);
        int32_t *mt_out = a.mt_start + kind * (nslots + 1);
        int32_t carry = 0;
        if (threadIdx.x == 0) hot_mtiles = 0;
        __syncthreads();
        for (int32_t base = 0; base < nslots; base += kTableThreads) {
            const int32_t pos = base + threadIdx.x;
            const int32_t F = pos < nslots && !ovf ? (sorted_rows[pos] + 31) >> 5 : 0;
            const int32_t mt = (F + fmax - 1) / fmax;
            int32_t chunk_total;
            const int32_t off = carry + block_exclusive_scan<kTableThreads / 64>(mt, wsum, &chunk_total);
            if (pos < nslots) mt_out[pos] = off;
            if (pos == hot) hot_mtiles = off;      // row-tiles of the busy slots
            carry += chunk_total;
        }
        __syncthreads();
        if (threadIdx.x == 0) mt_out[nslots] = carry;
        if (threadIdx.x == 0 && hot >= nslots) hot_mtiles = carry;
        mtotal[kind] = carry;
        __syncthreads();
        // rider units: one per tile of the busy slots while they last; a two-fragment slot
        // (4 nt units) is carried whole or not at all
        const int64_t nt = kind == 0 ? a.nt_gu : a.nt_dn;
        const int64_t units2 = (int64_t)ncold2 * 4 * nt, units = units2 + (int64_t)(ncold - ncold2) * 2 * nt;
        int64_t carried = fmax <= kRiderHostFrags ? min((int64_t)hot_mtiles * nt, units) : 0;
        if (nt > 0 && carried < units2) carried = carried / (4 * nt) * (4 * nt);
        riders[kind] = (int32_t)carried;
        __syncthreads();                           // hot_mtiles is rewritten by the next kind
    }
    if (threadIdx.x == 0) {
        a.ctrl[CTRL_HOT_SLOTS] = hot;
        a.ctrl[CTRL_LIVE_SLOTS] = live;
        a.ctrl[CTRL_COLD2_SLOTS] = ncold2;
        a.ctrl[CTRL_RIDERS_GATEUP] = riders[0];
        a.ctrl[CTRL_RIDERS_DOWN] = riders[1];
        a.ctrl[CTRL_MTILES] = mtotal[0];
    }
}

__global__ __launch_bounds__(256) void dispatch_kernel(DispatchArgs a) {
    if (blockIdx.x == gridDim.x - 1) {             // the extra workgroup: tile tables of the GEMMs
        build_tile_tables(a);
        return;
    }
    const craft_tables_header *hdr = reinterpret_cast<const craft_tables_header *>(a.tables);
    const int32_t *copies = a.tables + hdr->off_copies;
    const int32_t *efirst = a.tables + hdr->off_efirst;
    const int32_t *eslots = a.tables + hdr->off_eslots;
    const int64_t A = a.T * a.k;
    const int32_t per_block = kTokPerBlock * a.k;
    const int32_t *base = a.base + (int64_t)blockIdx.x * a.E;
    // several chunks of blocks: the prefixes are chunk-local, the chunk's base comes on top
    const int32_t *cbase = a.chunk_base ? a.chunk_base + (int64_t)(blockIdx.x / kScanChunk) * a.E : nullptr;
    for (int32_t i = threadIdx.x; i < per_block; i += blockDim.x) {
        const int64_t as = (int64_t)blockIdx.x * per_block + i;
        if (as >= A) break;
        const int32_t e = a.ids[as];
        const int32_t idx = base[e] + (cbase ? cbase[e] : 0) + (int32_t)a.lrank[as];   // i-th assignment of expert e
        const int32_t c = copies[e];
        const int32_t q = idx % c;
        const int32_t p = eslots[efirst[e] + q];
        const int32_t d = a.slot_off[p] + idx / c;
        a.dest[as] = d;
        a.src[d] = (int32_t)as;
        if (a.user_dest) a.user_dest[as] = d;
        if (a.user_src) a.user_src[d] = (int32_t)as;
    }
}

}  // namespace

hipError_t launch_scan(const ScanArgs &a, hipStream_t s) {
    // one chunk of token blocks: one workgroup does everything; more: one per chunk and 64 experts
    const unsigned chunks = (unsigned)((a.NB + kScanChunk - 1) / kScanChunk);
    const unsigned blocks = chunks <= 1 ? 1u : chunks * (unsigned)((a.E + 63) / 64);
    hipLaunchKernelGGL(scan_kernel, dim3(blocks), dim3(kScanThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_dispatch(const DispatchArgs &a, hipStream_t s) {
    if (a.T == 0) return hipSuccess;
    const int64_t nb = (a.T + kTokPerBlock - 1) / kTokPerBlock;
    hipLaunchKernelGGL(dispatch_kernel, dim3((unsigned)nb + 1), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace craft
