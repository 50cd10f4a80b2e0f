// Expert-load histogram over routing traces: the W[B][L][E] that Alg. 1 takes as input
// (Sec. 3.1 "expert load"), counted per profiling batch, layer and expert.
//
// HBM-bound: 4 bytes read per assignment, output negligible.  A workgroup streams one
// chunk of one (batch, layer) cell with 16-byte loads and counts into LDS.  Every wave
// keeps its own counters, and inside a wave the lanes are spread over several counter
// copies (lane mod copies), so the few hot experts of a Zipf-skewed trace do not
// serialise the LDS atomics of a whole wavefront.  At the end the copies are summed and
// the cell's counts are stored (one chunk per cell) or added with integer atomics
// (several chunks per cell, output cleared first); integer addition commutes, so the
// counts are exact either way.
#include <algorithm>

#include "kernels.h"

namespace craft {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kLdsWords = 16384;                 // 64 KiB of counters per workgroup
constexpr int64_t kChunkIds = 32768;             // assignments per workgroup (128 KiB)

__global__ void clear_counts_kernel(int64_t *p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

__global__ __launch_bounds__(kThreads) void expert_load_kernel(LoadArgs a, int32_t chunks,
                                                               int32_t ncopy) {
    extern __shared__ int32_t cnt[];             // [kWaves][ncopy][E]
    const int32_t E = a.E;
    const int64_t cell = blockIdx.x / chunks;    // = b * L + l
    const int32_t chunk = blockIdx.x % chunks;
    const int64_t b = cell / a.L;
    const int32_t l = (int32_t)(cell % a.L);
    const int64_t t0 = b * a.batch_tokens;
    const int64_t t1 = min(a.T, t0 + a.batch_tokens);
    const int64_t cell_ids = (t1 - t0) * a.k;
    const int64_t first = ((int64_t)l * a.T + t0) * a.k;      // index of the cell's first id
    const int64_t c0 = min(cell_ids, (int64_t)chunk * kChunkIds);
    const int64_t c1 = min(cell_ids, c0 + kChunkIds);

    const int words = kWaves * ncopy * E;
    for (int i = threadIdx.x; i < words; i += kThreads) cnt[i] = 0;
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t *mine = cnt + (wave * ncopy + (lane % ncopy)) * E;
    const int32_t *ids = a.ids + first;
    auto bump = [&](int32_t e) {
        if ((uint32_t)e < (uint32_t)E) atomicAdd(&mine[e], 1);
    };
    // scalar head up to 16-byte alignment, 16-byte body, scalar tail
    int64_t head = c0;
    while (head < c1 && ((first + head) & 3)) ++head;
    for (int64_t i = c0 + threadIdx.x; i < head; i += kThreads) bump(ids[i]);
    const int64_t nvec = (c1 - head) / 4;
    // the trace is read once: streaming loads
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const i32x4 *v = reinterpret_cast<const i32x4 *>(ids + head);
    int64_t i = threadIdx.x;
    for (; i + 3 * kThreads < nvec; i += 4 * kThreads) {
        const i32x4 q0 = __builtin_nontemporal_load(v + i), q1 = __builtin_nontemporal_load(v + i + kThreads),
                    q2 = __builtin_nontemporal_load(v + i + 2 * kThreads), q3 = __builtin_nontemporal_load(v + i + 3 * kThreads);
        bump(q0.x); bump(q0.y); bump(q0.z); bump(q0.w);
        bump(q1.x); bump(q1.y); bump(q1.z); bump(q1.w);
        bump(q2.x); bump(q2.y); bump(q2.z); bump(q2.w);
        bump(q3.x); bump(q3.y); bump(q3.z); bump(q3.w);
    }
    for (; i < nvec; i += kThreads) {
        const i32x4 q = __builtin_nontemporal_load(v + i);
        bump(q.x); bump(q.y); bump(q.z); bump(q.w);
    }
    for (int64_t j = head + nvec * 4 + threadIdx.x; j < c1; j += kThreads) bump(ids[j]);
    __syncthreads();

    int64_t *out = a.counts + cell * E;
    for (int e = threadIdx.x; e < E; e += kThreads) {
        int32_t s = 0;
        for (int c = 0; c < kWaves * ncopy; ++c) s += cnt[c * E + e];
        if (chunks == 1) out[e] = s;
        else if (s) atomicAdd(reinterpret_cast<unsigned long long *>(out + e), (unsigned long long)s);
    }
}

}  // namespace

// Sec. 4.3 step 1: the load window between two rebalancings grows by one forward's counts.
__global__ void load_accumulate_kernel(const int32_t *counts, int64_t n, int64_t *window) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) window[i] += counts[i];
}

hipError_t launch_load_accumulate(const int32_t *counts, int64_t n, int64_t *window, hipStream_t s) {
    hipLaunchKernelGGL(load_accumulate_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                       counts, n, window);
    return hipGetLastError();
}

hipError_t launch_expert_load(const LoadArgs &a, hipStream_t s) {
    const int64_t cells = a.B * a.L;
    if (cells == 0) return hipSuccess;
    const int64_t max_cell_ids = std::min(a.T, a.batch_tokens) * a.k;
    const int64_t chunks = std::max<int64_t>(1, (max_cell_ids + kChunkIds - 1) / kChunkIds);
    if (cells * chunks > 0x7fffffffLL) return hipErrorInvalidValue;
    int ncopy = kLdsWords / (kWaves * a.E);
    ncopy = std::max(1, std::min(8, ncopy));
    const size_t lds = (size_t)kWaves * ncopy * a.E * sizeof(int32_t);
    if (chunks > 1) {
        const int64_t n = cells * a.E;
        hipLaunchKernelGGL(clear_counts_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                           a.counts, n);
    }
    hipLaunchKernelGGL(expert_load_kernel, dim3((unsigned)(cells * chunks)), dim3(kThreads), lds, s,
                       a, (int32_t)chunks, ncopy);
    return hipGetLastError();
}

}  // namespace craft
