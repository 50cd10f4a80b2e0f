// Expert weights in 8 bits: OCP FP8 E4M3 codes with one fp32 scale per weight row, and their
// re-ordering into the stream the packed FFN kernels read (see ffn_packed.hip).  Not part of
// a forward: this is model loading.
//
// E4M3: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits; exponent field 0 is subnormal
// (mantissa / 8 * 2^-6); no infinities; S.1111.111 is NaN; the largest finite value is 448.
#include "kernels.h"

namespace craft {
namespace {

constexpr int kQuantThreads = 256;

__device__ __forceinline__ float bf16_value(unsigned short h) { return __uint_as_float((uint32_t)h << 16); }

// Nearest E4M3 magnitude to a >= 0, ties to the even mantissa, saturating at 448.  The value
// grid inside one binade is 2^(e-3), so the mantissa is a rounded quotient; below 2^-6 the
// grid is 2^-9 throughout.  rintf rounds halves to even, which is the rule for the code too
// (the last mantissa bit is the last bit of the code, and a carry into the next binade lands
// on its first, even, value).
__device__ __forceinline__ uint32_t e4m3_magnitude(float a) {
    if (!(a < 448.0f)) return 0x7e;
    if (a < 0.015625f) return (uint32_t)rintf(a * 512.0f);          // 0..8; 8 is the smallest normal
    const int e = (int)((__float_as_uint(a) >> 23) & 0xff) - 127;   // floor(log2 a), a is normal here
    const int n = (int)rintf(ldexpf(a, 3 - e));                     // 8..16
    const uint32_t code = n == 16 ? (uint32_t)(e + 8) << 3 : ((uint32_t)(e + 7) << 3) | (uint32_t)(n - 8);
    return code > 0x7e ? 0x7e : code;
}

// One workgroup per weight row: the row maximum, the scale, then the codes.
__global__ __launch_bounds__(kQuantThreads) void quantize_e4m3_kernel(const unsigned short *w, int32_t K,
                                                                      uint8_t *codes, float *scale) {
    __shared__ float part[kQuantThreads / 64];
    const int64_t r = blockIdx.x;
    const unsigned short *row = w + r * K;
    float amax = 0.0f;
    for (int k = threadIdx.x; k < K; k += kQuantThreads) amax = fmaxf(amax, fabsf(bf16_value(row[k])));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
    const float s = amax > 0.0f ? amax / 448.0f : 1.0f;
    if (threadIdx.x == 0) scale[r] = s;
    for (int k = threadIdx.x; k < K; k += kQuantThreads) {
        const float q = bf16_value(row[k]) / s;
        codes[r * K + k] = (uint8_t)(e4m3_magnitude(fabsf(q)) | (__float_as_uint(q) >> 31 << 7));
    }
}

// One 8-byte chunk of the packed stream per thread: the layout of the bf16 stream (step-major,
// 8 column groups per tile, two 16-row fragments per group, 64 lanes per fragment), with 8 codes
// where it has 8 bf16 values.
//   gate/up : group g = output columns 16g..16g+15; half 0 = gate rows 16g..16g+15, half 1 = the
//             up rows of the same columns
//   down    : group g = output columns 32g..32g+31; half h = down rows 32g+16h..+15
// Lane l of 32-wide step s holds row (l & 15) of its half, contraction elements 32s + 8(l>>4) .. +7.
__global__ void pack_e4m3_kernel(const uint8_t *ca, const uint8_t *cb, int rows, int K, int gc,
                                 int64_t nchunks, int ksteps, uint2 *out) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= nchunks) return;
    const int l = (int)(c & 63);
    const int h = (int)(c >> 6) & 1;
    const int64_t sg = c >> 7;
    const int64_t ngroups = nchunks / 128 / ksteps;
    const int s = (int)(sg / ngroups);
    const int64_t g = sg % ngroups;
    const int r = l & 15;
    const int k0 = 32 * s + 8 * (l >> 4);
    int64_t row;
    const uint8_t *src;
    if (gc == 16) { row = g * 16 + r; src = h ? cb : ca; }
    else { row = g * 32 + 16 * h + r; src = ca; }
    uint2 v = make_uint2(0, 0);
    if (row < rows && k0 < K) v = *reinterpret_cast<const uint2 *>(src + row * K + k0);
    out[c] = v;
}

__global__ void copy_scales_kernel(const float *a, const float *b, int n, float *out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = a[i];
    else if (b && i < 2 * n) out[i] = b[i - n];
}

}  // namespace

void packed_sizes_e4m3(int32_t H, int32_t I, size_t *gateup_bytes, size_t *down_bytes) {
    const size_t gu_groups = ((size_t)(I + 15) / 16 + 7) / 8 * 8, gu_steps = (size_t)(H + 255) / 256 * 16;
    const size_t dn_groups = ((size_t)(H + 31) / 32 + 7) / 8 * 8, dn_steps = (size_t)(I + 255) / 256 * 16;
    *gateup_bytes = gu_groups * gu_steps * 512 + (size_t)2 * I * sizeof(float);
    *down_bytes = dn_groups * dn_steps * 512 + (size_t)H * sizeof(float);
}

hipError_t launch_quantize_e4m3(const void *w, int64_t rows, int32_t K, uint8_t *codes, float *scale,
                                hipStream_t s) {
    hipLaunchKernelGGL(quantize_e4m3_kernel, dim3((unsigned)rows), dim3(kQuantThreads), 0, s,
                       static_cast<const unsigned short *>(w), K, codes, scale);
    return hipGetLastError();
}

hipError_t launch_pack_e4m3(int32_t H, int32_t I, const uint8_t *cg, const uint8_t *cu, const uint8_t *cd,
                            const float *sg, const float *su, const float *sd, void *pgu, void *pdn,
                            hipStream_t s) {
    size_t gub, dnb;
    packed_sizes_e4m3(H, I, &gub, &dnb);
    const size_t gu_stream = gub - (size_t)2 * I * sizeof(float), dn_stream = dnb - (size_t)H * sizeof(float);
    const int64_t c1 = (int64_t)(gu_stream / 8), c2 = (int64_t)(dn_stream / 8);
    hipLaunchKernelGGL(pack_e4m3_kernel, dim3((unsigned)((c1 + 255) / 256)), dim3(256), 0, s, cg, cu, I, H,
                       16, c1, (H + 255) / 256 * 8, static_cast<uint2 *>(pgu));
    hipLaunchKernelGGL(pack_e4m3_kernel, dim3((unsigned)((c2 + 255) / 256)), dim3(256), 0, s, cd, cd, H, I,
                       32, c2, (I + 255) / 256 * 8, static_cast<uint2 *>(pdn));
    float *gus = reinterpret_cast<float *>(static_cast<unsigned char *>(pgu) + gu_stream);
    float *dns = reinterpret_cast<float *>(static_cast<unsigned char *>(pdn) + dn_stream);
    hipLaunchKernelGGL(copy_scales_kernel, dim3((unsigned)((2 * I + 255) / 256)), dim3(256), 0, s, sg, su, I, gus);
    hipLaunchKernelGGL(copy_scales_kernel, dim3((unsigned)((H + 255) / 256)), dim3(256), 0, s, sd,
                       static_cast<const float *>(nullptr), H, dns);
    return hipGetLastError();
}

}  // namespace craft
