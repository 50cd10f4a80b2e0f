// Router softmax / top-k (Sec. 2.1: the gating network scores every expert and the
// top-K scores are activated), one 64-lane wavefront per token.
//
// A lane holds the scores of experts lane, lane+64, ... so a row is read with fully
// coalesced 256-byte requests.  The k picks are k wave-wide arg-max reductions over
// (score, expert id) with butterfly shuffles; scores are compared raw (never their
// exponentials) and equal scores resolve to the lower expert id.
//
// A workgroup covers 32 consecutive tokens.  While the picks are still in registers it
// also records, per expert, a 32-bit mask of the block's tokens that chose it: the number
// of set bits below a token's own bit is that assignment's rank among the block's
// assignments to the expert (experts of one token are distinct), and the population count
// is the block's contribution to the expert's load.
#include "kernels.h"

namespace craft {
namespace {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kTokPerWave = kTokPerBlock / kWavesPerBlock;
constexpr int kMaxE = 1024;

__device__ __forceinline__ bool beats(float va, int ia, float vb, int ib) {
    if (ia < 0) return false;
    if (ib < 0) return true;
    return va > vb || (va == vb && ia < ib);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

template <int VPT>
__global__ __launch_bounds__(kWave * kWavesPerBlock) void route_kernel(RouteArgs a) {
    __shared__ uint32_t mask[kMaxE];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const bool ranks = a.hist != nullptr;

    if (ranks) {
        for (int e = threadIdx.x; e < a.E; e += blockDim.x) mask[e] = 0u;
        if (a.ctrl && blockIdx.x == 0 && threadIdx.x < CTRL_WORDS) a.ctrl[threadIdx.x] = 0;
        __syncthreads();
    }

    int my_id[kTokPerWave];
#pragma unroll
    for (int it = 0; it < kTokPerWave; ++it) {
        my_id[it] = -1;
        const int tl = wave * kTokPerWave + it;
        const int64_t t = (int64_t)blockIdx.x * kTokPerBlock + tl;
        if (t >= a.T) continue;                       // uniform over the wave
        const float *row = a.logits + t * a.E;
        float v[VPT];
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int e = lane + kWave * i;
            v[i] = e < a.E ? row[e] : 0.0f;
        }
        uint32_t taken = 0u;
        float pick_v = 0.0f;
        int pick_i = -1;
        for (int j = 0; j < a.k; ++j) {
            float bv = 0.0f;
            int bi = -1;
#pragma unroll
            for (int i = 0; i < VPT; ++i) {
                const int e = lane + kWave * i;
                if (e < a.E && !((taken >> i) & 1u) && (bi < 0 || v[i] > bv)) { bv = v[i]; bi = e; }
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const float ov = __shfl_xor(bv, off, kWave);
                const int oi = __shfl_xor(bi, off, kWave);
                if (beats(ov, oi, bv, bi)) { bv = ov; bi = oi; }
            }
            if ((bi & (kWave - 1)) == lane) taken |= 1u << (bi >> 6);
            if (lane == j) { pick_v = bv; pick_i = bi; }
        }
        // softmax weight of the picks; the first pick carries the row maximum
        const float mx = __shfl(pick_v, 0, kWave);
        const float ex = lane < a.k ? expf(pick_v - mx) : 0.0f;
        float den;
        if (a.renorm) {
            den = wave_sum(ex);
        } else {
            float s = 0.0f;
#pragma unroll
            for (int i = 0; i < VPT; ++i)
                if (lane + kWave * i < a.E) s += expf(v[i] - mx);
            den = wave_sum(s);
        }
        if (lane < a.k) {
            a.ids[t * a.k + lane] = pick_i;
            a.w[t * a.k + lane] = ex / den;
            my_id[it] = pick_i;
            if (ranks) atomicOr(&mask[pick_i], 1u << tl);
        }
    }
    if (!ranks) return;
    __syncthreads();
#pragma unroll
    for (int it = 0; it < kTokPerWave; ++it) {
        const int tl = wave * kTokPerWave + it;
        const int64_t t = (int64_t)blockIdx.x * kTokPerBlock + tl;
        if (t < a.T && lane < a.k)
            a.lrank[t * a.k + lane] = (uint8_t)__popc(mask[my_id[it]] & ((1u << tl) - 1u));
    }
    int32_t *hrow = a.hist + (int64_t)blockIdx.x * a.E;
    for (int e = threadIdx.x; e < a.E; e += blockDim.x) hrow[e] = __popc(mask[e]);
}

__global__ void clear_ctrl_kernel(int32_t *ctrl) {
    if (threadIdx.x < CTRL_WORDS) ctrl[threadIdx.x] = 0;
}

}  // namespace

hipError_t launch_route(const RouteArgs &a, hipStream_t s) {
    if (a.T == 0) {
        // nothing to route; the control words still have to be cleared for the next stage
        // (a kernel rather than a memset node, so the call stays safe to capture in a graph)
        if (a.ctrl) hipLaunchKernelGGL(clear_ctrl_kernel, dim3(1), dim3(64), 0, s, a.ctrl);
        return hipGetLastError();
    }
    const int64_t nb = (a.T + kTokPerBlock - 1) / kTokPerBlock;
    dim3 grid((unsigned)nb), block(kWave * kWavesPerBlock);
    const int vpt = (a.E + kWave - 1) / kWave;
    if (vpt <= 1) hipLaunchKernelGGL(route_kernel<1>, grid, block, 0, s, a);
    else if (vpt <= 2) hipLaunchKernelGGL(route_kernel<2>, grid, block, 0, s, a);
    else if (vpt <= 4) hipLaunchKernelGGL(route_kernel<4>, grid, block, 0, s, a);
    else if (vpt <= 6) hipLaunchKernelGGL(route_kernel<6>, grid, block, 0, s, a);
    else if (vpt <= 8) hipLaunchKernelGGL(route_kernel<8>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(route_kernel<16>, grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace craft
