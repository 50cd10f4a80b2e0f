// Gating-network scores, the input of top-K routing (Sec. 2.1).  The paper leaves the form of
// the network open; this is the usual linear gate,
//   logits[t][e] = sum_h x[t][h] * Wr[e][h],
// both operands contiguous along the contraction, fp32 accumulation, fp32 scores.  The top-k
// step consumes these scores exactly as it consumes scores handed in from outside.
//
// A skinny GEMM: few output columns (E = 128 .. 384), so the tokens' activations are what
// has to cross HBM (once) and the gate's weights are re-read from L2 by every workgroup.
// bf16: a workgroup of four waves takes NXF fragments of 32 tokens against up to 512 experts
// (more experts: further workgroups along y); wave w owns the blocks of 32 experts w, w + 4, ..
// Both operands are staged through LDS in slabs of 64 (rows padded to 144 bytes, two stages,
// one barrier per slab) and D slabs travel in registers ahead of the one being multiplied
// (v_mfma_f32_32x32x16_bf16).  The activations feed the MFMA's row operand and the gate rows
// its column operand, so that for each accumulator element lanes 0-31 hold 32 consecutive
// experts of one token: stores are 128 contiguous bytes.
// What bounds it: every workgroup pulls the whole gate out of L2, so T H 2 (1 + E / tokens
// per workgroup) bytes move from L2 into the CUs, at the 11-12 TB/s the chip sustains there
// with every CU pulling.  Taller workgroups move less but there are only T / 128 of them, so
// with a workspace the contraction is split over up to 8 workgroups per tile: each writes
// its partial scores and a second kernel adds them in ascending order of the split (a fixed
// order: the result does not depend on scheduling).  Gate rows loaded straight into
// registers in operand layout (32-byte pieces of 32 rows per request) measured slower.
// fp32: one thread per score, a plain chain of fused multiply-adds (small configurations).
#include "ffn_common.h"

namespace craft {
namespace {

constexpr int GK = 64;                  // contraction slab
constexpr int GROWB = GK * 2 + 16;      // padded LDS row, bytes
typedef unsigned int gu32x4_t __attribute__((ext_vector_type(4)));
typedef const gu32x4_t __attribute__((address_space(1))) *gchunk_t;

template <int NB, int NXF, int D>
__global__ __launch_bounds__(256) void router_logits_bf16_kernel(RouterArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char gate_smem[];
    constexpr int STAGEB = (NXF * 32 + NB * 128) * GROWB;  // activations [NXF * 32] rows, gate [NB * 128]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lr = tid >> 3, kc = tid & 7;                 // row (plus 32 i) and 16-byte chunk staged
    const int frag_off = (lane & 31) * GROWB + (lane >> 5) * 16;
    const int64_t t0 = (int64_t)blockIdx.x * (NXF * 32);
    const int e0 = blockIdx.y * (NB * 128);
    const int hchunks = a.H >> 3;                          // 16-byte chunks per row
    // this workgroup's share of the contraction: slabs kbeg .. kbeg + nk - 1 (nk may be 0)
    const int nk_all = (a.H + GK - 1) / GK;
    const int per = (nk_all + a.nsplit - 1) / a.nsplit;
    const int kbeg = min(nk_all, (int)blockIdx.z * per);
    const int nk = min(nk_all, kbeg + per) - kbeg;
    float *dst = a.nsplit > 1 ? a.part + (int64_t)blockIdx.z * a.T * a.E : a.logits;

    // rows past the end are clamped into the matrix (their results are not stored)
    gchunk_t xrow[NXF], wrow[NB * 4];
#pragma unroll
    for (int i = 0; i < NXF; ++i)
        xrow[i] = (gchunk_t)a.x + min(t0 + lr + 32 * i, a.T - 1) * hchunks;
#pragma unroll
    for (int j = 0; j < NB * 4; ++j)
        wrow[j] = (gchunk_t)a.w + (int64_t)min(e0 + lr + 32 * j, a.E - 1) * hchunks;

    f32x16_t acc[NB][NXF];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int g = 0; g < NXF; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][g][v] = 0.0f;

    gu32x4_t xr[D][NXF], wr[D][NB * 4];
    const gu32x4_t zero = {0u, 0u, 0u, 0u};
    // Slab ks -> register set d.  A chunk past the end of the rows is read from inside the
    // rows instead and replaced by zeros when it goes to LDS: touching the value here would
    // make the wave wait for the load on the spot.
#define GATE_REQUEST(d, ks)                                                              \
    {                                                                                    \
        const int c = min((ks) * (GK / 8) + kc, hchunks - 1);                            \
        _Pragma("unroll") for (int i = 0; i < NXF; ++i) xr[d][i] = xrow[i][c];           \
        _Pragma("unroll") for (int j = 0; j < NB * 4; ++j) wr[d][j] = wrow[j][c];        \
    }
    // no branch around a request, here or in the loop: the count of loads in flight has to be
    // the same on every path for the waits to let D slabs stay outstanding (past the last
    // slab the last one is requested again and never used)
#pragma unroll
    for (int d = 0; d < D; ++d) GATE_REQUEST(d, min(kbeg + d, nk_all - 1))
    for (int ks0 = 0; ks0 < nk; ks0 += 2 * D) {
#pragma unroll
        for (int dd = 0; dd < 2 * D; ++dd) {               // 2 D slabs per trip: set and stage are static
            const int ks = ks0 + dd;
            if (ks >= nk) break;
            const int d = dd % D;
            unsigned char *xs = gate_smem + (dd & 1) * STAGEB;
            unsigned char *ws = xs + NXF * 32 * GROWB;
            const bool in = (kbeg + ks) * (GK / 8) + kc < hchunks;
#pragma unroll
            for (int i = 0; i < NXF; ++i)
                *reinterpret_cast<gu32x4_t *>(xs + (lr + 32 * i) * GROWB + kc * 16) = in ? xr[d][i] : zero;
#pragma unroll
            for (int j = 0; j < NB * 4; ++j)
                *reinterpret_cast<gu32x4_t *>(ws + (lr + 32 * j) * GROWB + kc * 16) = in ? wr[d][j] : zero;
            // one barrier per slab: the other stage is rewritten only after every wave has
            // passed this one, that is, has finished reading it
            __syncthreads();
            GATE_REQUEST(d, min(kbeg + ks + D, nk_all - 1))
#pragma unroll
            for (int step = 0; step < GK / 16; ++step) {
                bf16x8_t xa[NXF];
#pragma unroll
                for (int g = 0; g < NXF; ++g)
                    xa[g] = *reinterpret_cast<const bf16x8_t *>(xs + g * 32 * GROWB + frag_off + step * 32);
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const bf16x8_t wb = *reinterpret_cast<const bf16x8_t *>(
                        ws + (b * 4 + wave) * 32 * GROWB + frag_off + step * 32);
#pragma unroll
                    for (int g = 0; g < NXF; ++g)
                        acc[b][g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[g], wb, acc[b][g], 0, 0, 0);
                }
            }
        }
    }
#undef GATE_REQUEST

    // accumulator element v of lane l: token row (v/4)*8 + (l>>5)*4 + v%4 of the fragment,
    // expert (l & 31) of the block
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int e = e0 + (b * 4 + wave) * 32 + (lane & 31);
#pragma unroll
        for (int g = 0; g < NXF; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t t = t0 + g * 32 + (v / 4) * 8 + (lane >> 5) * 4 + v % 4;
                if (t < a.T && e < a.E) dst[t * a.E + e] = acc[b][g][v];
            }
    }
}

// logits = sum of the partial scores, in ascending order of the split
__global__ __launch_bounds__(256) void router_reduce_kernel(const float *part, int nsplit, int64_t n, float *logits) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    float s = part[i];
    for (int z = 1; z < nsplit; ++z) s += part[(int64_t)z * n + i];
    logits[i] = s;
}

__global__ __launch_bounds__(256) void router_logits_f32_kernel(RouterArgs a) {
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= a.T * a.E) return;
    const float *x = static_cast<const float *>(a.x) + (o / a.E) * a.H;
    const float *w = static_cast<const float *>(a.w) + (o % a.E) * a.H;
    float s = 0.0f;
    for (int h = 0; h < a.H; ++h) s = fmaf(x[h], w[h], s);
    a.logits[o] = s;
}

template <int NB, int NXF, int D>
hipError_t launch_bf16(const RouterArgs &a, hipStream_t s) {
    constexpr size_t lds = (size_t)2 * (NXF * 32 + NB * 128) * GROWB;
    static_assert(lds <= 160 * 1024, "two stages have to fit the CU's LDS");
    static bool raised = false;                            // more than the default 64 KB of LDS
    if (!raised && lds > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(router_logits_bf16_kernel<NB, NXF, D>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const dim3 grid((unsigned)((a.T + NXF * 32 - 1) / (NXF * 32)), (unsigned)((a.E + NB * 128 - 1) / (NB * 128)),
                    (unsigned)a.nsplit);
    hipLaunchKernelGGL((router_logits_bf16_kernel<NB, NXF, D>), grid, dim3(256), lds, s, a);
    if (a.nsplit > 1) {
        const int64_t n = a.T * a.E;
        hipLaunchKernelGGL(router_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                           a.part, a.nsplit, n, a.logits);
    }
    return hipGetLastError();
}

}  // namespace

// Tile height (32-token fragments per workgroup) and split of the contraction for a shape.
// Without a workspace: short tiles, as many as there are CUs if possible.  With one: the
// tallest tile the registers allow, and as many splits as bring the workgroups up to the CU
// count (at most 8, at least 4 slabs each).
void router_logits_shape(int64_t T, int32_t H, int32_t E, int32_t num_cu, bool workspace, int *nxf, int *nsplit) {
    const int nb = E > 512 ? 4 : (E + 127) / 128;
    *nsplit = 1;
    if (!workspace || nb > 3) {
        *nxf = nb <= 3 && (T + 63) / 64 >= (int64_t)num_cu ? 2 : 1;
        return;
    }
    *nxf = 4;
    const int64_t tiles = (T + 127) / 128 * ((E + nb * 128 - 1) / (nb * 128));
    const int nk = (H + GK - 1) / GK;
    int sp = 1;
    while (sp < 8 && tiles * sp * 2 <= num_cu && nk / (sp * 2) >= 4) sp *= 2;
    *nsplit = sp;
}

hipError_t launch_router_logits(const RouterArgs &a, hipStream_t s) {
    if (a.T == 0) return hipSuccess;
    if (a.dtype == CRAFT_F32) {
        const int64_t n = a.T * a.E;
        hipLaunchKernelGGL(router_logits_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a);
        return hipGetLastError();
    }
    const int nb = a.E > 512 ? 4 : (a.E + 127) / 128;      // blocks of 32 experts per wave
    int nxf, nsplit;
    router_logits_shape(a.T, a.H, a.E, a.num_cu, a.part != nullptr, &nxf, &nsplit);
    RouterArgs b = a;
    b.nsplit = nsplit;
    switch (nb * 16 + nxf) {
        case 1 * 16 + 1: return launch_bf16<1, 1, 4>(b, s);
        case 1 * 16 + 2: return launch_bf16<1, 2, 4>(b, s);
        case 1 * 16 + 4: return launch_bf16<1, 4, 4>(b, s);
        case 2 * 16 + 1: return launch_bf16<2, 1, 4>(b, s);
        case 2 * 16 + 2: return launch_bf16<2, 2, 4>(b, s);
        case 2 * 16 + 4: return launch_bf16<2, 4, 3>(b, s);
        case 3 * 16 + 1: return launch_bf16<3, 1, 3>(b, s);
        case 3 * 16 + 2: return launch_bf16<3, 2, 3>(b, s);
        case 3 * 16 + 4: return launch_bf16<3, 4, 1>(b, s);
        default: return launch_bf16<4, 1, 3>(b, s);
    }
}

}  // namespace craft
