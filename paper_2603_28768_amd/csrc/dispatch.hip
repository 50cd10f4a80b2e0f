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

// Exclusive scan of n values produced by `get(i)`, written through `put(i, prefix)`;
// returns the total to every thread.  Each thread owns a contiguous run of items.
template <typename Get, typename Put>
__device__ int32_t block_exclusive_scan(int32_t n, int32_t *sh /*[kScanThreads]*/, Get get, Put put) {
    const int tid = threadIdx.x;
    const int32_t per = (n + kScanThreads - 1) / kScanThreads;
    const int32_t lo = min(n, tid * per), hi = min(n, lo + per);
    int32_t sum = 0;
    for (int32_t i = lo; i < hi; ++i) sum += get(i);
    sh[tid] = sum;
    __syncthreads();
    for (int off = 1; off < kScanThreads; off <<= 1) {
        int32_t v = tid >= off ? sh[tid - off] : 0;
        __syncthreads();
        sh[tid] += v;
        __syncthreads();
    }
    const int32_t total = sh[kScanThreads - 1];
    int32_t run = sh[tid] - sum;
    for (int32_t i = lo; i < hi; ++i) {
        const int32_t v = get(i);
        put(i, run);
        run += v;
    }
    __syncthreads();
    return total;
}

// One workgroup per 64 experts.  Wave w owns a contiguous range of blocks; a lane owns one
// expert.  Pass 1 sums the range, the waves' sums are prefix-combined through LDS, pass 2
// rewrites the per-block counts as exclusive prefixes.  The workgroup that finishes last
// (ticket counter) derives everything that needs all counts: rows per slot, slot offsets,
// the rank's row count and the row-tile table of the grouped GEMMs.
__global__ __launch_bounds__(kScanThreads) void scan_kernel(ScanArgs a) {
    __shared__ int32_t sh[kScanThreads];
    __shared__ int32_t part[kScanWaves][64];
    __shared__ int32_t last_flag;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int e = blockIdx.x * 64 + lane;
    const int rows_per_wave = (a.NB + kScanWaves - 1) / kScanWaves;
    const int b0 = min(a.NB, wave * rows_per_wave), b1 = min(a.NB, b0 + rows_per_wave);

    int32_t sum = 0;
    if (e < a.E)
        for (int b = b0; b < b1; ++b) sum += a.hist[(int64_t)b * a.E + e];
    part[wave][lane] = sum;
    __syncthreads();
    int32_t before = 0, total = 0;
    for (int w = 0; w < kScanWaves; ++w) {
        const int32_t v = part[w][lane];
        if (w < wave) before += v;
        total += v;
    }
    if (e < a.E) {
        int32_t run = before;
        for (int b = b0; b < b1; ++b) {
            int32_t *p = a.hist + (int64_t)b * a.E + e;
            const int32_t v = *p;
            *p = run;
            run += v;
        }
        if (wave == 0) {
            a.counts[e] = total;
            if (a.user_counts) a.user_counts[e] = total;
        }
    }

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

    const craft_tables_header *hdr = reinterpret_cast<const craft_tables_header *>(a.tables);
    const int32_t *copies = a.tables + hdr->off_copies;
    const int32_t *slot_expert = a.tables + hdr->off_slot_expert;
    const int32_t *slot_copy = a.tables + hdr->off_slot_copy;
    const int32_t *counts = a.counts;

    // rows of slot p: tokens i < n of its expert with i mod c == q
    auto slot_rows = [&](int32_t p) -> int32_t {
        const int32_t ex = slot_expert[p];
        const int32_t n = __hip_atomic_load(counts + ex, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int32_t c = copies[ex], q = slot_copy[p];
        return n > q ? (n - q + c - 1) / c : 0;
    };
    const int32_t all = block_exclusive_scan(
        a.S, sh, slot_rows, [&](int32_t p, int32_t pre) {
            a.slot_off[p] = pre;
            if (a.user_slot_off) a.user_slot_off[p] = pre;
        });
    for (int32_t p = threadIdx.x; p < a.S; p += kScanThreads) {
        const int32_t r = slot_rows(p);
        a.slot_cnt[p] = r;
        if (a.user_slot_cnt) a.user_slot_cnt[p] = r;
    }
    if (threadIdx.x == 0) {
        a.slot_off[a.S] = all;
        if (a.user_slot_off) a.user_slot_off[a.S] = all;
    }
    // this rank's rows; refuse the batch when they exceed the staging buffers
    __shared__ int32_t rank_rows, overflow;
    if (threadIdx.x == 0) {
        int32_t r = 0;
        for (int32_t p = a.s_lo; p < a.s_hi; ++p) r += slot_rows(p);
        rank_rows = r;
        overflow = (int64_t)r > a.max_rows;
    }
    __syncthreads();
    const bool ovf = overflow != 0;
    const int32_t nslots = a.s_hi - a.s_lo;
    const int32_t mtiles = block_exclusive_scan(
        nslots, sh,
        [&](int32_t s) -> int32_t { return ovf ? 0 : (slot_rows(a.s_lo + s) + a.bm - 1) / a.bm; },
        [&](int32_t s, int32_t pre) { a.mt_start[s] = pre; });
    if (threadIdx.x == 0) {
        a.mt_start[nslots] = mtiles;
        a.ctrl[CTRL_ROWS] = rank_rows;
        a.ctrl[CTRL_OVERFLOW] = overflow;
        a.ctrl[CTRL_MTILES] = mtiles;
        a.ctrl[CTRL_TICKET] = 0;
    }
}

__global__ __launch_bounds__(256) void dispatch_kernel(DispatchArgs a) {
    const craft_tables_header *hdr = reinterpret_cast<const craft_tables_header *>(a.tables);
    const int32_t *copies = a.tables + hdr->off_copies;
    const int32_t *efirst = a.tables + hdr->off_efirst;
    const int32_t *eslots = a.tables + hdr->off_eslots;
    const int64_t A = a.T * a.k;
    const int32_t per_block = kTokPerBlock * a.k;
    const int32_t *base = a.base + (int64_t)blockIdx.x * a.E;
    for (int32_t i = threadIdx.x; i < per_block; i += blockDim.x) {
        const int64_t as = (int64_t)blockIdx.x * per_block + i;
        if (as >= A) break;
        const int32_t e = a.ids[as];
        const int32_t idx = base[e] + (int32_t)a.lrank[as];    // i-th assignment of expert e
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
    const unsigned blocks = (unsigned)((a.E + 63) / 64);
    hipLaunchKernelGGL(scan_kernel, dim3(blocks), dim3(kScanThreads), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_dispatch(const DispatchArgs &a, hipStream_t s) {
    if (a.T == 0) return hipSuccess;
    const int64_t nb = (a.T + kTokPerBlock - 1) / kTokPerBlock;
    hipLaunchKernelGGL(dispatch_kernel, dim3((unsigned)nb), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace craft
