// Gating-network scores (Sec. 2.1: for each token the gating network computes a score for
// each expert).  The paper gives no form for the network; this is the usual linear gate,
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
// with every CU pulling.  Taller workgroups would move less but leave CUs idle (T / 128
// workgroups) and serialise LDS traffic and MFMAs inside one wave per SIMD; they measured
// slower, as did gate rows loaded straight into registers in operand layout (32-byte pieces
// of 32 rows per request).  Splitting the contraction over workgroups, with partial scores
// in a workspace and a second pass adding them in a fixed order, is the way past this.
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
    const int nk = (a.H + GK - 1) / GK;
    const int hchunks = a.H >> 3;                          // 16-byte chunks per row

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
    for (int d = 0; d < D; ++d) GATE_REQUEST(d, min(d, nk - 1))
    for (int ks0 = 0; ks0 < nk; ks0 += 2 * D) {
#pragma unroll
        for (int dd = 0; dd < 2 * D; ++dd) {               // 2 D slabs per trip: set and stage are static
            const int ks = ks0 + dd;
            if (ks >= nk) break;
            const int d = dd % D;
            unsigned char *xs = gate_smem + (dd & 1) * STAGEB;
            unsigned char *ws = xs + NXF * 32 * GROWB;
            const bool in = ks * (GK / 8) + kc < hchunks;
#pragma unroll
            for (int i = 0; i < NXF; ++i)
                *reinterpret_cast<gu32x4_t *>(xs + (lr + 32 * i) * GROWB + kc * 16) = in ? xr[d][i] : zero;
#pragma unroll
            for (int j = 0; j < NB * 4; ++j)
                *reinterpret_cast<gu32x4_t *>(ws + (lr + 32 * j) * GROWB + kc * 16) = in ? wr[d][j] : zero;
            // one barrier per slab: the other stage is rewritten only after every wave has
            // passed this one, that is, has finished reading it
            __syncthreads();
            GATE_REQUEST(d, min(ks + D, nk - 1))
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
                if (t < a.T && e < a.E) a.logits[t * a.E + e] = acc[b][g][v];
            }
    }
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
    const dim3 grid((unsigned)((a.T + NXF * 32 - 1) / (NXF * 32)), (unsigned)((a.E + NB * 128 - 1) / (NB * 128)));
    hipLaunchKernelGGL((router_logits_bf16_kernel<NB, NXF, D>), grid, dim3(256), lds, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_router_logits(const RouterArgs &a, hipStream_t s) {
    if (a.T == 0) return hipSuccess;
    if (a.dtype == CRAFT_F32) {
        const int64_t n = a.T * a.E;
        hipLaunchKernelGGL(router_logits_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a);
        return hipGetLastError();
    }
    const int nb = a.E > 512 ? 4 : (a.E + 127) / 128;      // blocks of 32 experts per wave
    const bool two = (a.T + 63) / 64 >= (int64_t)a.num_cu;  // two token fragments if every CU still gets work
    switch (nb) {
        case 1: return two ? launch_bf16<1, 2, 4>(a, s) : launch_bf16<1, 1, 4>(a, s);
        case 2: return two ? launch_bf16<2, 2, 4>(a, s) : launch_bf16<2, 1, 4>(a, s);
        case 3: return two ? launch_bf16<3, 2, 3>(a, s) : launch_bf16<3, 1, 3>(a, s);
        default: return launch_bf16<4, 1, 3>(a, s);
    }
}

}  // namespace craft
