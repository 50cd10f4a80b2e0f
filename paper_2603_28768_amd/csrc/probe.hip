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

}  // namespace

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
