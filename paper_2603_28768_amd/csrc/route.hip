// Router softmax / top-k: the top-K routing step of the MoE layer of Sec. 2.1.
//
// A token is handled by one 16-lane DPP row of a 64-lane wavefront, so a wave routes four
// tokens at once and every cross-lane step is a row-local DPP move (quad permutes and
// row mirrors), not an LDS permute.  A lane holds the scores of experts 4*lane..4*lane+3,
// +64, +128, ... (16-byte loads; a token's row is read as contiguous 256-byte pieces).
// Each of the k picks is an arg-max over (score, expert id): first inside the lane in
// ascending expert order, then a four-step butterfly over the row.  Scores are compared
// raw, never their exponentials, and equal scores resolve to the lower expert id.
//
// A workgroup of eight waves covers 32 consecutive tokens.  While the picks are still in
// registers it also records, per expert, a 32-bit mask of the block's tokens that chose it:
// the number of set bits below a token's own bit is that assignment's rank among the
// block's assignments to the expert (experts of one token are distinct), and the
// population count is the block's contribution to the expert's load.
#include "kernels.h"

namespace craft {
namespace {

constexpr int kThreads = 16 * kTokPerBlock;   // a 16-lane row per token of the block
constexpr int kMaxE = 1024;
constexpr int kMaxPickSlots = 4;     // k <= 64 picks, 16 lanes per token

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
// lane exchange patterns that together reach every lane of a 16-lane row
constexpr int kXor1 = 0xB1, kXor2 = 0x4E, kHalfMirror = 0x141, kMirror = 0x140;

__device__ __forceinline__ bool beats(float va, int ia, float vb, int ib) {
    return va > vb || (va == vb && ia < ib);
}

template <int CTRL>
__device__ __forceinline__ void argmax_step(float &v, int &i) {
    const float ov = dpp_f<CTRL>(v);
    const int oi = dpp_i<CTRL>(i);
    if (beats(ov, oi, v, i)) { v = ov; i = oi; }
}

__device__ __forceinline__ float row_sum(float v) {
    v += dpp_f<kXor1>(v);
    v += dpp_f<kXor2>(v);
    v += dpp_f<kHalfMirror>(v);
    v += dpp_f<kMirror>(v);
    return v;
}

// NQ = 16-byte score chunks per lane (each chunk = 4 experts; a row covers 64 experts per chunk)
template <int NQ>
__global__ __launch_bounds__(kThreads) void route_kernel(RouteArgs a) {
    __shared__ uint32_t mask[kMaxE];
    const int tid = threadIdx.x;
    const int sub = tid & 15;                      // lane inside the token's row
    const bool ranks = a.hist != nullptr;
    // 16-byte loads need every row 16-byte aligned; otherwise the scores are read one by one
    const bool vec_ok = (a.E & 3) == 0 && (reinterpret_cast<uintptr_t>(a.logits) & 15) == 0;

    if (ranks) {
        for (int e = tid; e < a.E; e += kThreads) mask[e] = 0u;
        if (a.ctrl && blockIdx.x == 0 && tid < CTRL_WORDS) a.ctrl[tid] = 0;
        __syncthreads();
    }

    int my_id[kMaxPickSlots];
    const int tl = tid >> 4;                       // token inside the block
    const int64_t t = (int64_t)blockIdx.x * kTokPerBlock + tl;
    {
#pragma unroll
        for (int s = 0; s < kMaxPickSlots; ++s) my_id[s] = -1;
        const bool live = t < a.T;                 // uniform over the row
        const float *row = a.logits + (live ? t : 0) * a.E;

        // Experts past E and experts already picked hold -inf: a finite score always beats
        // them (k <= E, and scores are finite by contract).
        constexpr float kGone = -__builtin_huge_valf();
        float v[NQ][4];
        auto load_scores = [&]() {
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int e0 = q * 64 + sub * 4;
                if (vec_ok && e0 + 3 < a.E) {
                    const float4 f = *reinterpret_cast<const float4 *>(row + e0);
                    v[q][0] = f.x; v[q][1] = f.y; v[q][2] = f.z; v[q][3] = f.w;
                } else {
#pragma unroll
                    for (int c = 0; c < 4; ++c) v[q][c] = e0 + c < a.E ? row[e0 + c] : kGone;
                }
            }
        };
        load_scores();

        float pick_v[kMaxPickSlots];
        float first_v = 0.0f;
#pragma unroll
        for (int s = 0; s < kMaxPickSlots; ++s) {
            pick_v[s] = 0.0f;
            const int jn = min(16, a.k - s * 16);  // picks that land in slot s
            for (int j = 0; j < jn; ++j) {
                // the lane's best: a tournament in ascending expert order, the later entry
                // winning only when strictly greater, so equal scores keep the lower id
                float tv[NQ * 4];
                int ti[NQ * 4];
#pragma unroll
                for (int q = 0; q < NQ; ++q)
#pragma unroll
                    for (int c = 0; c < 4; ++c) { tv[q * 4 + c] = v[q][c]; ti[q * 4 + c] = q * 64 + sub * 4 + c; }
#pragma unroll
                for (int width = 1; width < NQ * 4; width *= 2)
#pragma unroll
                    for (int i = 0; i + width < NQ * 4; i += 2 * width)
                        if (tv[i + width] > tv[i]) { tv[i] = tv[i + width]; ti[i] = ti[i + width]; }
                float bv = tv[0];
                int bi = ti[0];
                argmax_step<kXor1>(bv, bi);
                argmax_step<kXor2>(bv, bi);
                argmax_step<kHalfMirror>(bv, bi);
                argmax_step<kMirror>(bv, bi);
                // the owner retires the pick; lane j of the row keeps it for the output
#pragma unroll
                for (int q = 0; q < NQ; ++q)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (bi == q * 64 + sub * 4 + c) v[q][c] = kGone;
                if (j == sub) { pick_v[s] = bv; my_id[s] = bi; }
                if (s == 0 && j == 0) first_v = bv;       // the row maximum
            }
        }
        // softmax weight of the picks
        float ex[kMaxPickSlots], part = 0.0f;
#pragma unroll
        for (int s = 0; s < kMaxPickSlots; ++s) {
            ex[s] = s * 16 + sub < a.k ? expf(pick_v[s] - first_v) : 0.0f;
            part += ex[s];
        }
        if (!a.renorm) {
            load_scores();                         // the picks were blanked out: read the row again
            part = 0.0f;
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (q * 64 + sub * 4 + c < a.E) part += expf(v[q][c] - first_v);
        }
        const float den = row_sum(part);
        if (live) {
#pragma unroll
            for (int s = 0; s < kMaxPickSlots; ++s) {
                const int j = s * 16 + sub;
                if (j < a.k) {
                    a.ids[t * a.k + j] = my_id[s];
                    a.w[t * a.k + j] = ex[s] / den;
                    if (ranks) atomicOr(&mask[my_id[s]], 1u << tl);
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < kMaxPickSlots; ++s) my_id[s] = -1;
        }
    }
    if (!ranks) return;
    __syncthreads();
#pragma unroll
    for (int s = 0; s < kMaxPickSlots; ++s) {
        const int j = s * 16 + sub;
        if (t < a.T && j < a.k)
            a.lrank[t * a.k + j] = (uint8_t)__popc(mask[my_id[s]] & ((1u << tl) - 1u));
    }
    int32_t *hrow = a.hist + (int64_t)blockIdx.x * a.E;
    for (int e = tid; e < a.E; e += kThreads) hrow[e] = __popc(mask[e]);
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
    dim3 grid((unsigned)nb), block(kThreads);
    const int nq = (a.E + 63) / 64;
    if (nq <= 1) hipLaunchKernelGGL(route_kernel<1>, grid, block, 0, s, a);
    else if (nq <= 2) hipLaunchKernelGGL(route_kernel<2>, grid, block, 0, s, a);
    else if (nq <= 4) hipLaunchKernelGGL(route_kernel<4>, grid, block, 0, s, a);
    else if (nq <= 6) hipLaunchKernelGGL(route_kernel<6>, grid, block, 0, s, a);
    else if (nq <= 8) hipLaunchKernelGGL(route_kernel<8>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(route_kernel<16>, grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace craft
