// Grouped SwiGLU expert FFN of one rank (Sec. 2.1: each expert is an up-projection, a
// non-linearity and a down-projection; here down(silu(gate x) * up x)).
//
// Two grouped GEMMs over the rank's slots, both "NT" (activation rows and weight rows are
// contiguous along the contraction):
//   gate/up : act[r][i] = silu(sum_h x[r][h] Wg[i][h]) * (sum_h x[r][h] Wu[i][h])
//   down    : y[r][h]   = sum_i act[r][i] Wd[h][i]
//
// Work is cut into tiles of (slot, column tile, row tile).  Slots differ wildly in rows
// under skewed routing, so the tile list is data dependent: the scan kernel leaves a
// prefix table of row tiles per slot in device memory and a persistent grid walks the
// flattened list; a slot with no rows contributes no tile, a slot with few rows one
// (ragged) row tile per column tile.  Row tiles of the same (slot, column tile) are
// adjacent in the list and the workgroup-to-tile mapping keeps neighbours on one XCD, so
// a weight tile is fetched from HBM once and re-read from that XCD's L2.
//
// bf16 path: 128 x 128 x 64 tiles on v_mfma_f32_32x32x16_bf16, fp32 accumulation, both
// operands staged through LDS (double buffered, rows padded to 144 bytes so 16-byte
// fragment reads spread over all banks).  The weight rows feed the MFMA's row operand and
// the activation rows its column operand, so that a lane ends up with four consecutive
// output columns of one activation row (an 8-byte store).  For gate/up the 128 weight rows
// of a tile are 64 gate rows and the matching 64 up rows; each wave holds gate and up
// accumulators for the same outputs and applies SwiGLU in registers.  The gate/up GEMM
// reads its rows straight from x through the dispatch permutation (no staged copy).
//
// fp32 path: a plain LDS-tiled FMA kernel with the same tile list (small configurations).
#include "ffn_common.h"

namespace craft {
namespace {

// ------------------------------------------------------------------ bf16 / MFMA
constexpr int BM = kFragsBf16 * 32; // most activation rows per tile
constexpr int BK = 64;            // contraction slab
constexpr int ROWB = BK * 2 + 16; // padded LDS row, bytes
constexpr int TILEB = 128 * ROWB; // one operand tile
constexpr int STAGEB = 2 * TILEB;

template <bool GATEUP>
__global__ __launch_bounds__(256, 2) void ffn_bf16_kernel(FfnArgs a) {
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * STAGEB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave & 1, wm = wave >> 1;
    const int K = GATEUP ? a.H : a.I;              // contraction length
    const int N = GATEUP ? a.I : a.H;              // output columns
    constexpr int BN = GATEUP ? 64 : 128;          // output columns per tile
    const int nt = (N + BN - 1) / BN;
    const int nk = (K + BK - 1) / BK;
    const int32_t *mt_start = a.mt_start + (GATEUP ? 0 : a.nslots + 1);
    const int64_t total = (int64_t)mt_start[a.nslots] * nt;
    const int32_t lo_pos = a.slot_off[a.s_lo];
    const unsigned short *xin = static_cast<const unsigned short *>(GATEUP ? a.x : a.act);

    const int lr = tid >> 3;                       // row handled when loading (plus 32*i)
    const int kc = tid & 7;                        // 16-byte chunk inside the slab
    const int nf0 = GATEUP ? wn * 32 : wn * 64;    // weight-row fragments of this wave
    const int nf1 = GATEUP ? 64 + wn * 32 : wn * 64 + 32;
    const int mf0 = wm * 64, mf1 = wm * 64 + 32;   // activation-row fragments
    const int frag_off = (lane & 31) * ROWB + (lane >> 5) * 16;

    for (int64_t w = xcd_major_id(); w < total; w += gridDim.x) {
        const Tile t = decode_tile(a, mt_start, w, nt, BN, GATEUP ? a.frags_gu : a.frags_dn);
        const unsigned short *wa = static_cast<const unsigned short *>(
            GATEUP ? a.w_gate[t.slot] : a.w_down[t.slot]);
        const unsigned short *wb = GATEUP ? static_cast<const unsigned short *>(a.w_up[t.slot]) : wa;

        const unsigned short *xp[4], *wp[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = lr + 32 * i;
            const int rr = min(r, t.rows - 1);
            const int32_t pos = t.pos0 + t.m0 + rr;
            if (GATEUP) xp[i] = xin + (int64_t)(a.src[pos] / a.k) * K + kc * 8;
            else xp[i] = xin + (int64_t)(pos - lo_pos) * K + kc * 8;
            int wr;
            const unsigned short *wbase;
            if (GATEUP) { wr = t.n0 + (r & 63); wbase = r < 64 ? wa : wb; }
            else { wr = t.n0 + r; wbase = wa; }
            wr = min(wr, N - 1);
            wp[i] = wbase + (int64_t)wr * K + kc * 8;
        }

        f32x16_t acc[2][2];
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[f][g][v] = 0.0f;

        uint4 xr[4], wr4[4];
        auto load_slab = [&](int ks) {
            const int koff = ks * BK;
            const bool ok = koff + kc * 8 < K;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                xr[i] = ok ? *reinterpret_cast<const uint4 *>(xp[i] + koff) : make_uint4(0, 0, 0, 0);
                wr4[i] = ok ? *reinterpret_cast<const uint4 *>(wp[i] + koff) : make_uint4(0, 0, 0, 0);
            }
        };
        auto store_slab = [&](int stage) {
            unsigned char *ws = smem + stage * STAGEB, *xs = ws + TILEB;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int off = (lr + 32 * i) * ROWB + kc * 16;
                *reinterpret_cast<uint4 *>(ws + off) = wr4[i];
                *reinterpret_cast<uint4 *>(xs + off) = xr[i];
            }
        };

        load_slab(0);
        store_slab(0);
        __syncthreads();
        for (int ks = 0; ks < nk; ++ks) {
            const int cur = ks & 1;
            if (ks + 1 < nk) load_slab(ks + 1);
            const unsigned char *ws = smem + cur * STAGEB, *xs = ws + TILEB;
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) {
                const int ko = frag_off + kk * 32;
                const bf16x8_t w0 = *reinterpret_cast<const bf16x8_t *>(ws + nf0 * ROWB + ko);
                const bf16x8_t w1 = *reinterpret_cast<const bf16x8_t *>(ws + nf1 * ROWB + ko);
                const bf16x8_t x0 = *reinterpret_cast<const bf16x8_t *>(xs + mf0 * ROWB + ko);
                const bf16x8_t x1 = *reinterpret_cast<const bf16x8_t *>(xs + mf1 * ROWB + ko);
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w0, x0, acc[0][0], 0, 0, 0);
                acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w0, x1, acc[0][1], 0, 0, 0);
                acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1, x0, acc[1][0], 0, 0, 0);
                acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1, x1, acc[1][1], 0, 0, 0);
            }
            if (ks + 1 < nk) store_slab(cur ^ 1);
            __syncthreads();
        }

        // epilogue: lane holds, for activation row (lane & 31) of each row fragment, output
        // columns vg*8 + (lane>>5)*4 + 0..3 of each weight fragment
        unsigned short *outp = static_cast<unsigned short *>(GATEUP ? a.act : a.y);
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            const int m = (g ? mf1 : mf0) + (lane & 31);
            if (m >= t.rows) continue;
            unsigned short *orow = outp + (int64_t)(t.pos0 + t.m0 + m - lo_pos) * N;
#pragma unroll
            for (int vg = 0; vg < 4; ++vg) {
                const int nloc = vg * 8 + (lane >> 5) * 4;
                if (GATEUP) {
                    const int col = t.n0 + wn * 32 + nloc;
                    if (col < N) {
                        uint32_t h[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            h[c] = bf16_rne(silu(acc[0][g][vg * 4 + c]) * acc[1][g][vg * 4 + c]);
                        *reinterpret_cast<uint2 *>(orow + col) =
                            make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                    }
                } else {
#pragma unroll
                    for (int f = 0; f < 2; ++f) {
                        const int col = t.n0 + (f ? nf1 : nf0) + nloc;
                        if (col < N) {
                            uint32_t h[4];
#pragma unroll
                            for (int c = 0; c < 4; ++c) h[c] = bf16_rne(acc[f][g][vg * 4 + c]);
                            *reinterpret_cast<uint2 *>(orow + col) =
                                make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                        }
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------ fp32
constexpr int FM = kFragsF32 * 32;  // rows per tile
constexpr int FN = 32;            // output columns per tile
constexpr int FK = 32;            // contraction slab

template <bool GATEUP>
__global__ __launch_bounds__(256) void ffn_f32_kernel(FfnArgs a) {
    __shared__ float xs[FM][FK + 1];
    __shared__ float was[FN][FK + 1];
    __shared__ float wbs[FN][FK + 1];
    const int tid = threadIdx.x, tx = tid & 31, ty = tid >> 5;
    const int K = GATEUP ? a.H : a.I;
    const int N = GATEUP ? a.I : a.H;
    const int nt = (N + FN - 1) / FN;
    const int32_t *mt_start = a.mt_start + (GATEUP ? 0 : a.nslots + 1);
    const int64_t total = (int64_t)mt_start[a.nslots] * nt;
    const int32_t lo_pos = a.slot_off[a.s_lo];
    const float *xin = static_cast<const float *>(GATEUP ? a.x : a.act);

    for (int64_t w = xcd_major_id(); w < total; w += gridDim.x) {
        const Tile t = decode_tile(a, mt_start, w, nt, FN, GATEUP ? a.frags_gu : a.frags_dn);
        const float *wa = static_cast<const float *>(GATEUP ? a.w_gate[t.slot] : a.w_down[t.slot]);
        const float *wb = GATEUP ? static_cast<const float *>(a.w_up[t.slot]) : wa;
        const float *xrow[4], *warow[4], *wbrow[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = ty + 8 * i;
            const int32_t pos = t.pos0 + t.m0 + min(r, t.rows - 1);
            xrow[i] = GATEUP ? xin + (int64_t)(a.src[pos] / a.k) * K : xin + (int64_t)(pos - lo_pos) * K;
            const int wr = min(t.n0 + r, N - 1);
            warow[i] = wa + (int64_t)wr * K;
            wbrow[i] = wb + (int64_t)wr * K;
        }
        float ga[4] = {0, 0, 0, 0}, ub[4] = {0, 0, 0, 0};
        for (int k0 = 0; k0 < K; k0 += FK) {
            const bool ok = k0 + tx < K;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = ty + 8 * i;
                xs[r][tx] = ok ? xrow[i][k0 + tx] : 0.0f;
                was[r][tx] = ok ? warow[i][k0 + tx] : 0.0f;
                if (GATEUP) wbs[r][tx] = ok ? wbrow[i][k0 + tx] : 0.0f;
            }
            __syncthreads();
#pragma unroll 8
            for (int kk = 0; kk < FK; ++kk) {
                const float wv = was[tx][kk];
                const float uv = GATEUP ? wbs[tx][kk] : 0.0f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float xv = xs[ty * 4 + j][kk];
                    ga[j] += xv * wv;
                    if (GATEUP) ub[j] += xv * uv;
                }
            }
            __syncthreads();
        }
        float *outp = static_cast<float *>(GATEUP ? a.act : a.y);
        const int col = t.n0 + tx;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = ty * 4 + j;
            if (m < t.rows && col < N) {
                const float g = ga[j];
                const float val = GATEUP ? (g / (1.0f + expf(-g))) * ub[j] : g;
                outp[(int64_t)(t.pos0 + t.m0 + m - lo_pos) * N + col] = val;
            }
        }
    }
}

template <bool GATEUP>
hipError_t launch_ffn(const FfnArgs &a, hipStream_t s) {
    if (a.nslots <= 0 || a.max_rows <= 0) return hipSuccess;
    const int K = GATEUP ? a.H : a.I, N = GATEUP ? a.I : a.H;
    (void)K;
    if (a.dtype == CRAFT_BF16) {
        const int bn = GATEUP ? 64 : 128;
        const int64_t nt = (N + bn - 1) / bn;
        const int64_t bound = (a.max_rows / BM + a.nslots) * nt;    // most tiles any batch can have
        int64_t grid = std::min<int64_t>(bound, (int64_t)a.num_cu * 2);
        grid = std::max<int64_t>(8, (grid + 7) / 8 * 8);
        hipLaunchKernelGGL(ffn_bf16_kernel<GATEUP>, dim3((unsigned)grid), dim3(256), 0, s, a);
    } else {
        const int64_t nt = (N + FN - 1) / FN;
        const int64_t bound = (a.max_rows / FM + a.nslots) * nt;
        int64_t grid = std::min<int64_t>(bound, (int64_t)a.num_cu * 8);
        grid = std::max<int64_t>(8, (grid + 7) / 8 * 8);
        hipLaunchKernelGGL(ffn_f32_kernel<GATEUP>, dim3((unsigned)grid), dim3(256), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gateup(const FfnArgs &a, hipStream_t s) { return launch_ffn<true>(a, s); }
hipError_t launch_down(const FfnArgs &a, hipStream_t s) { return launch_ffn<false>(a, s); }

}  // namespace craft
