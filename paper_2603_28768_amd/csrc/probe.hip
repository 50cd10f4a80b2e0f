// Two measurement probes, so that a benchmark can state the box's own ceilings next to the
// published ones: a plain copy of known size (also the kernel of known traffic that memory
// counters are scaled against) and a register-only loop of bf16 MFMAs.  Neither is part of
// the forward.
#include "ffn_common.h"

namespace craft {
namespace {

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// dst[i] = src[i] in 16-byte pieces, consecutive lanes on consecutive pieces.
__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4_t *src, u32x4_t *dst, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

// Every workgroup reads the whole buffer `passes` times, 16 bytes per lane and eight requests
// in flight per lane, each workgroup starting at another place.  With a buffer that fits the
// L2 of every XCD (and not the 32 KB L1 of a CU) this is the rate at which all CUs together
// can pull data out of L2; the XOR of everything read goes to `sink`.
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4_t *src, int64_t n, int passes, uint32_t *sink) {
    u32x4_t acc = {0u, 0u, 0u, 0u};
    // workgroups that may share a compute unit (every 256th) start an eighth of the buffer apart,
    // neighbours 8 KiB apart: no two of them walk the same lines at the same time, so the 32 KB
    // L1 of a compute unit serves none of this
    const int64_t start = ((int64_t)(blockIdx.x >> 8) * (n >> 3) + (int64_t)(blockIdx.x & 255) * 512) % n;
    for (int p = 0; p < passes; ++p)
        for (int64_t base = 0; base < n; base += 8 * 256) {
            u32x4_t v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                int64_t i = start + base + u * 256 + threadIdx.x;
                i -= i >= n ? n : 0;
                v[u] = src[i];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) acc ^= v[u];
        }
    sink[(int64_t)blockIdx.x * blockDim.x + threadIdx.x] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}

// Every wave issues iters x 4 independent v_mfma_f32_32x32x16_bf16 on operands it made up
// itself; nothing is loaded.  The sums go to `sink` so the loop cannot be dropped.
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float *sink) {
    bf16x8_t a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(float)((threadIdx.x + i) & 3);
        b[i] = (__bf16)(0.25f * (float)((threadIdx.x * 3 + i) & 3));
    }
    f32x16_t acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[j][v];
    sink[(int64_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The matrix rate as a function of what the operands hold and of the instruction's shape.  The
// chip lowers its clock under the power the matrix pipelines draw, and that power depends on
// how many operand bits change from one instruction to the next: a loop over zeros or small
// integers says little about a GEMM on real activations.  Every wave keeps the FFN tile's
// register shape (2 weight x 8 activation fragments per step, 256 accumulator registers, two
// steps of distinct operands taken in turn) and issues the same floating-point work per
// iteration with either shape; nothing is loaded.
//   data 0: zeros;  1: the values 1.0 and 1.5;  2: random signs and mantissas, exponents spread
//   over 2^-8 .. 2^-1 (products and sums stay far from overflow for any iteration count)
static __device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}
static __device__ __forceinline__ bf16x8_t probe_operand(uint32_t seed, int data) {
    u32x4_t r;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t h = probe_hash(seed * 4 + i);
        uint32_t lo = 0, hi = 0;
        if (data == 1) { lo = 0x3f80 + ((h & 1) << 6); hi = 0x3f80 + ((h >> 1 & 1) << 6); }
        if (data == 2) { lo = (h & 0x807f) | ((119 + (h >> 8 & 7)) << 7); hi = ((h >> 16) & 0x807f) | ((119 + (h >> 24 & 7)) << 7); }
        r[i] = lo | (hi << 16);
    }
    return __builtin_bit_cast(bf16x8_t, r);
}
template <int SHAPE>   // 0: v_mfma_f32_32x32x16_bf16, 1: v_mfma_f32_16x16x32_bf16
__global__ __launch_bounds__(256, 1) void probe_mfma_operands_kernel(int iters, int data, float *sink) {
    bf16x8_t w[2][2], x[2][8];
    const uint32_t t = blockIdx.x * 256 + threadIdx.x;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int n = 0; n < 2; ++n) w[s][n] = probe_operand(t * 64 + s * 16 + n, data);
#pragma unroll
        for (int g = 0; g < 8; ++g) x[s][g] = probe_operand(t * 64 + s * 16 + 2 + g, data);
    }
    float sum = 0.0f;
    if (SHAPE == 0) {
        f32x16_t acc[2][8];
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int g = 0; g < 8; ++g) acc[n][g] = (f32x16_t)(0.0f);
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int n = 0; n < 2; ++n)
#pragma unroll
                    for (int g = 0; g < 8; ++g)
                        acc[n][g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[s][n], x[s][g], acc[n][g], 0, 0, 0);
        }
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int g = 0; g < 8; ++g)
#pragma unroll
                for (int v = 0; v < 16; ++v) sum += acc[n][g][v];
    } else {
        // a 32 x 32 block of outputs over 32 contraction elements: four products of 16 x 16 x 32
        f32x4_t acc[2][8][4];
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int g = 0; g < 8; ++g)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[n][g][q] = (f32x4_t)(0.0f);
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int n = 0; n < 2; ++n)
#pragma unroll
                for (int g = 0; g < 8; ++g) {
                    acc[n][g][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[0][n], x[0][g], acc[n][g][0], 0, 0, 0);
                    acc[n][g][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[0][n], x[1][g], acc[n][g][1], 0, 0, 0);
                    acc[n][g][2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[1][n], x[0][g], acc[n][g][2], 0, 0, 0);
                    acc[n][g][3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[1][n], x[1][g], acc[n][g][3], 0, 0, 0);
                }
        }
#pragma unroll
        for (int n = 0; n < 2; ++n)
#pragma unroll
            for (int g = 0; g < 8; ++g)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int v = 0; v < 4; ++v) sum += acc[n][g][q][v];
    }
    sink[t] = sum;
}

}  // namespace

hipError_t launch_probe_mfma_operands(int32_t shape, int32_t data, int32_t blocks, int32_t iters, float *sink,
                                      hipStream_t s) {
    if (shape == 0) hipLaunchKernelGGL(probe_mfma_operands_kernel<0>, dim3((unsigned)blocks), dim3(256), 0, s, iters, data, sink);
    else hipLaunchKernelGGL(probe_mfma_operands_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, s, iters, data, sink);
    return hipGetLastError();
}

hipError_t launch_probe_copy(const void *src, void *dst, int64_t bytes, int32_t num_cu, hipStream_t s) {
    const int64_t n = bytes / 16;
    const int64_t blocks = std::min<int64_t>((n + 255) / 256, (int64_t)num_cu * 16);
    hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<const u32x4_t *>(src), static_cast<u32x4_t *>(dst), n);
    return hipGetLastError();
}

hipError_t launch_probe_read(const void *src, int64_t bytes, int32_t passes, int32_t blocks, uint32_t *sink,
                             hipStream_t s) {
    hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<const u32x4_t *>(src), bytes / 16, passes, sink);
    return hipGetLastError();
}

hipError_t launch_probe_mfma(int32_t blocks, int32_t iters, float *sink, hipStream_t s) {
    hipLaunchKernelGGL(probe_mfma_kernel, dim3((unsigned)blocks), dim3(256), 0, s, iters, sink);
    return hipGetLastError();
}

}  // namespace craft
