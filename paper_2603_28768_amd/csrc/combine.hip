// Gather-weighted combine: the last step of the MoE layer of Sec. 2.1, each token's sum of
// its experts' outputs scaled by the routing weights.  One 64-lane wavefront per token; a lane owns 16-byte column chunks of the
// row.  Only assignments whose dispatched position falls inside this rank's row range
// contribute, added in ascending j with fp32 accumulation; there are no atomics, so the
// result does not depend on scheduling.  Tokens with no assignment on the rank get zeros.
#include <hip/hip_bf16.h>

#include "kernels.h"

namespace craft {
namespace {

// A 16-byte piece of a row as it is loaded, and how it unpacks to fp32 / packs from it.
template <typename T> struct Chunk;
template <> struct Chunk<float> {
    static constexpr int N = 4;
    __device__ static void unpack(const uint4 &q, float (&v)[4]) {
        v[0] = __uint_as_float(q.x); v[1] = __uint_as_float(q.y);
        v[2] = __uint_as_float(q.z); v[3] = __uint_as_float(q.w);
    }
    __device__ static uint4 pack(const float (&v)[4]) {
        return make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]),
                          __float_as_uint(v[3]));
    }
};
template <> struct Chunk<__hip_bfloat16> {
    static constexpr int N = 8;
    __device__ static void unpack(const uint4 &q, float (&v)[8]) {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static uint32_t rne(float f) {       // fp32 -> bf16 bits, nearest even
        const uint32_t u = __float_as_uint(f);
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    }
    __device__ static uint4 pack(const float (&v)[8]) {
        uint4 q;
        q.x = rne(v[0]) | (rne(v[1]) << 16);
        q.y = rne(v[2]) | (rne(v[3]) << 16);
        q.z = rne(v[4]) | (rne(v[5]) << 16);
        q.w = rne(v[6]) | (rne(v[7]) << 16);
        return q;
    }
};

template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs a) {
    constexpr int N = Chunk<T>::N;
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= a.T) return;
    const int32_t lo = a.slot_off[a.s_lo], hi = a.slot_off[a.s_hi];
    const bool dead = a.ctrl[CTRL_OVERFLOW] != 0;
    int32_t d = -1;
    float wj = 0.0f;
    if (lane < a.k) {
        d = a.dest[t * a.k + lane];
        wj = a.w[t * a.k + lane];
    }
    const bool mine = !dead && lane < a.k && d >= lo && d < hi;
    const unsigned long long live = __ballot(mine);
    const T *y = static_cast<const T *>(a.y);
    T *out = static_cast<T *>(a.out) + t * a.H;
    // The chunk loop is uniform over the wave (shuffles need every lane); a lane past the end
    // of the row only skips its loads and its store.  A lane owns U chunks of the row and the
    // rows of up to G assignments are requested together before any of them is added (in
    // ascending j, as always): what a wave takes is a chain of memory latencies, one per round
    // of requests, and a token of the busiest rank has several of its experts there.
    constexpr int U = 8, G = 4;
    for (int base = 0; base < a.H; base += 64 * N * U) {
        int c0[U];
        bool inside[U];
        float acc[U][N];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            c0[u] = base + (u * 64 + lane) * N;
            inside[u] = c0[u] < a.H;
#pragma unroll
            for (int i = 0; i < N; ++i) acc[u][i] = 0.0f;
        }
        unsigned long long m = live;
        while (m) {
            const T *row[G];
            float wv[G];
            int n = 0;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                row[g] = y;
                wv[g] = 0.0f;
                if (m) {
                    const int j = __ffsll((long long)m) - 1;
                    m &= m - 1;
                    row[g] = y + (int64_t)(__shfl(d, j, 64) - lo) * a.H;
                    wv[g] = __shfl(wj, j, 64);
                    n = g + 1;
                }
            }
            uint4 raw[G][U];
#pragma unroll
            for (int g = 0; g < G; ++g)
                if (g < n) {
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        raw[g][u] = inside[u] ? *reinterpret_cast<const uint4 *>(row[g] + c0[u])
                                              : make_uint4(0, 0, 0, 0);
                }
#pragma unroll
            for (int g = 0; g < G; ++g)
                if (g < n) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        float v[N];
                        Chunk<T>::unpack(raw[g][u], v);
#pragma unroll
                        for (int i = 0; i < N; ++i) acc[u][i] += wv[g] * v[i];
                    }
                }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (inside[u]) {
                // written once and not read again by this launch: a streaming store
                typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
                const uint4 q = Chunk<T>::pack(acc[u]);
                const u32x4 v = {q.x, q.y, q.z, q.w};
                __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(out + c0[u]));
            }
    }
}

}  // namespace

hipError_t launch_combine(const CombineArgs &a, hipStream_t s) {
    if (a.T == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((a.T + 3) / 4);
    if (a.dtype == CRAFT_F32)
        hipLaunchKernelGGL(combine_kernel<float>, dim3(blocks), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(combine_kernel<__hip_bfloat16>, dim3(blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace craft
