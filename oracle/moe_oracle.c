/*
 * CPU checker for one expert-parallel rank's MoE layer under a replication plan.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, written from the definitions; used by
 * the test-suite, the smoke check and the benchmark's CPU-baseline leg.  It
 * shares no code with the HIP library and the library never calls it.
 *
 * Floating point is accumulated in double throughout (the method fixes no
 * precision for the reference; inputs arrive as float values that are exactly
 * representable in their storage type).
 *
 * What is computed, and where the paper defines it:
 *   oracle_router_logits Sec. 2.1 (routing): per-token expert scores from a gating network
 *                        whose form the paper leaves open; read as the usual linear
 *                        gate, score[t][e] = x[t] . W_r[e], no bias.
 *   oracle_route         Sec. 2.1 (routing): top-K of the scores per token, with the
 *                        routing weights of the K picked.
 *   oracle_expert_load   Sec. 3.1 "expert load", the W[b][l][e] input of Alg. 1: routed
 *                        assignments per expert, per batch and layer.
 *   oracle_dispatch      Sec. 1 / Alg. 1: a replicated expert's tokens are spread
 *                        evenly over its copies; the i-th token of expert e goes
 *                        to copy i mod c_e.
 *   oracle_ffn_rows      Sec. 2.1: expert = up-projection, non-linearity,
 *                        down-projection (SwiGLU form: down(silu(gate x) * up x)).
 *   oracle_combine       Sec. 2.1: expert outputs aggregated into a weighted sum.
 *   oracle_e4m3_value, oracle_quantize_e4m3
 *                        not in the paper: 8-bit storage of expert weights (OCP FP8
 *                        E4M3: 1 sign, 4 exponent bits with bias 7, 3 mantissa bits,
 *                        no infinities, S.1111.111 = NaN, largest finite 448), one
 *                        scale per weight row.  Replication memory is what the paper
 *                        trades against balance; halving the bytes of a replica is
 *                        the adjacent lever.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Sec. 2.1 gating network, linear form: logits[t][e] = sum_h x[t][h] * Wr[e][h], the sum
 * taken in double over h ascending and rounded once to float.  x [T][H], Wr [E][H]. */
int oracle_router_logits(const float *x, const float *Wr, int64_t T, int32_t H, int32_t E,
                         float *logits)
{
    if (T < 0 || H <= 0 || E <= 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int32_t e = 0; e < E; ++e) {
            const float *a = x + t * H, *b = Wr + (int64_t)e * H;
            double s = 0.0;
            for (int32_t h = 0; h < H; ++h) s += (double)a[h] * (double)b[h];
            logits[t * E + e] = (float)s;
        }
    return 0;
}

/* Sec. 2.1 router.  ids[t][j] = expert with the (j+1)-th largest raw score of
 * token t (equal scores: lower expert id first).  w[t][j] = softmax probability
 * of that expert over all E scores, divided by the sum over the k picked when
 * renorm != 0.  Returns 0, or -1 on bad sizes. */
int oracle_route(const float *logits, int64_t T, int32_t E, int32_t k, int32_t renorm,
                 int32_t *ids, float *w)
{
    if (T < 0 || E <= 0 || k <= 0 || k > E) return -1;
    unsigned char *taken = (unsigned char *)malloc((size_t)E);
    double *p = (double *)malloc(sizeof(double) * (size_t)E);
    if (!taken || !p) { free(taken); free(p); return -2; }
    for (int64_t t = 0; t < T; ++t) {
        const float *l = logits + t * E;
        memset(taken, 0, (size_t)E);
        for (int32_t j = 0; j < k; ++j) {
            int32_t best = -1;
            for (int32_t e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || l[e] > l[best]) best = e;
            }
            taken[best] = 1;
            ids[t * k + j] = best;
        }
        double mx = (double)l[0];
        for (int32_t e = 1; e < E; ++e) if ((double)l[e] > mx) mx = (double)l[e];
        double den = 0.0;
        for (int32_t e = 0; e < E; ++e) { p[e] = exp((double)l[e] - mx); den += p[e]; }
        double picked = 0.0;
        for (int32_t j = 0; j < k; ++j) picked += p[ids[t * k + j]] / den;
        for (int32_t j = 0; j < k; ++j) {
            double pj = p[ids[t * k + j]] / den;
            w[t * k + j] = (float)(renorm ? pj / picked : pj);
        }
    }
    free(taken); free(p);
    return 0;
}

/* Sec. 3.1 / Alg. 1 input.  ids is [L][T][k]; counts is [B][L][E] with
 * B = ceil(T / batch_tokens), zeroed here.  Returns -1 on an id outside [0,E). */
int oracle_expert_load(const int32_t *ids, int32_t L, int64_t T, int32_t k, int32_t E,
                       int64_t batch_tokens, int64_t *counts)
{
    if (L <= 0 || T < 0 || k <= 0 || E <= 0 || batch_tokens <= 0) return -1;
    int64_t B = (T + batch_tokens - 1) / batch_tokens;
    memset(counts, 0, sizeof(int64_t) * (size_t)(B * L * E));
    for (int32_t l = 0; l < L; ++l)
        for (int64_t t = 0; t < T; ++t)
            for (int32_t j = 0; j < k; ++j) {
                int32_t e = ids[((int64_t)l * T + t) * k + j];
                if (e < 0 || e >= E) return -1;
                counts[((t / batch_tokens) * L + l) * E + e] += 1;
            }
    return 0;
}

/* Replica-aware dispatch.  Slots are the physical expert copies of the layer in
 * plan order; slot_expert[p] names the expert held by slot p; the copies of an
 * expert are its slots in ascending slot number.  Assignments a = t*k+j are
 * visited in order; the i-th one that names expert e is appended to the list of
 * e's copy number (i mod c_e).  The slot lists, concatenated in slot order, are
 * src; dest is the inverse.  slot_cnt[S], slot_off[S+1].
 * Returns 0, -1 on an id out of range or an expert without a slot. */
int oracle_dispatch(const int32_t *ids, int64_t A, int32_t E, int32_t S,
                    const int32_t *slot_expert,
                    int32_t *dest, int32_t *src, int32_t *slot_cnt, int32_t *slot_off)
{
    int rc = 0;
    int32_t *copies = (int32_t *)calloc((size_t)E, sizeof(int32_t));
    int32_t *first = (int32_t *)malloc(sizeof(int32_t) * (size_t)(E + 1));
    int32_t *slots_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)S);
    int64_t *seen = (int64_t *)calloc((size_t)E, sizeof(int64_t));
    int32_t *where = (int32_t *)malloc(sizeof(int32_t) * (size_t)(A > 0 ? A : 1));
    int32_t *fill = (int32_t *)malloc(sizeof(int32_t) * (size_t)S);
    if (!copies || !first || !slots_of || !seen || !where || !fill) { rc = -2; goto done; }

    for (int32_t p = 0; p < S; ++p) {
        if (slot_expert[p] < 0 || slot_expert[p] >= E) { rc = -1; goto done; }
        copies[slot_expert[p]] += 1;
    }
    first[0] = 0;
    for (int32_t e = 0; e < E; ++e) first[e + 1] = first[e] + copies[e];
    {   /* slots_of[first[e] + q] = q-th slot (ascending) that holds expert e */
        int32_t *n = (int32_t *)calloc((size_t)E, sizeof(int32_t));
        if (!n) { rc = -2; goto done; }
        for (int32_t p = 0; p < S; ++p) {
            int32_t e = slot_expert[p];
            slots_of[first[e] + n[e]] = p;
            n[e] += 1;
        }
        free(n);
    }
    memset(slot_cnt, 0, sizeof(int32_t) * (size_t)S);
    for (int64_t a = 0; a < A; ++a) {
        int32_t e = ids[a];
        if (e < 0 || e >= E || copies[e] == 0) { rc = -1; goto done; }
        int64_t i = seen[e]++;
        int32_t p = slots_of[first[e] + (int32_t)(i % copies[e])];
        where[a] = p;
        slot_cnt[p] += 1;
    }
    slot_off[0] = 0;
    for (int32_t p = 0; p < S; ++p) slot_off[p + 1] = slot_off[p] + slot_cnt[p];
    for (int32_t p = 0; p < S; ++p) fill[p] = slot_off[p];
    for (int64_t a = 0; a < A; ++a) {
        int32_t d = fill[where[a]]++;
        src[d] = (int32_t)a;
        dest[a] = d;
    }
done:
    free(copies); free(first); free(slots_of); free(seen); free(where); free(fill);
    return rc;
}

/* One expert's SwiGLU feed-forward over `rows` input rows.
 * X [rows][H], Wg/Wu [I][H], Wd [H][I] (all contraction-contiguous), Y [rows][H].
 *   g_i = sum_h X[r][h] Wg[i][h];  u_i likewise;  a_i = g_i / (1 + exp(-g_i)) * u_i;
 *   Y[r][h] = sum_i a_i Wd[h][i].                                                  */
int oracle_ffn_rows(const float *X, int64_t rows, int32_t H, int32_t I,
                    const float *Wg, const float *Wu, const float *Wd, double *Y)
{
    if (rows < 0 || H <= 0 || I <= 0) return -1;
    int rc = 0;
#pragma omp parallel
    {
        double *act = (double *)malloc(sizeof(double) * (size_t)I);
        if (!act) {
#pragma omp atomic write
            rc = -2;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < rows; ++r) {
            if (!act) continue;
            const float *x = X + r * H;
            for (int32_t i = 0; i < I; ++i) {
                const float *wg = Wg + (int64_t)i * H, *wu = Wu + (int64_t)i * H;
                double g = 0.0, u = 0.0;
                for (int32_t h = 0; h < H; ++h) {
                    g += (double)x[h] * (double)wg[h];
                    u += (double)x[h] * (double)wu[h];
                }
                act[i] = g / (1.0 + exp(-g)) * u;
            }
            for (int32_t h = 0; h < H; ++h) {
                const float *wd = Wd + (int64_t)h * I;
                double y = 0.0;
                for (int32_t i = 0; i < I; ++i) y += act[i] * (double)wd[i];
                Y[r * H + h] = y;
            }
        }
        free(act);
    }
    return rc;
}

/* Weighted sum of one rank's expert outputs.  Y [M][H] holds the rank's rows in
 * dispatch order (row d - lo of Y is global position d); an assignment belongs
 * to the rank when lo <= dest < lo + M.  out [T][H] is fully written (zeros for
 * tokens none of whose experts live on the rank); terms are added j ascending. */
int oracle_combine(const double *Y, int64_t M, int64_t lo, const int32_t *dest, const float *w,
                   int64_t T, int32_t k, int32_t H, double *out)
{
    if (T < 0 || k <= 0 || H <= 0 || M < 0) return -1;
    for (int64_t t = 0; t < T; ++t) {
        double *o = out + t * H;
        for (int32_t h = 0; h < H; ++h) o[h] = 0.0;
        for (int32_t j = 0; j < k; ++j) {
            int64_t d = dest[t * k + j];
            if (d < lo || d >= lo + M) continue;
            const double *y = Y + (d - lo) * H;
            double wj = (double)w[t * k + j];
            for (int32_t h = 0; h < H; ++h) o[h] += wj * y[h];
        }
    }
    return 0;
}

/* Value of an E4M3 code, from the format's definition: exponent field 0 is subnormal,
 * mantissa / 8 * 2^-6; otherwise (1 + mantissa / 8) * 2^(exponent - 7).  NaN codes give NaN. */
double oracle_e4m3_value(uint8_t code)
{
    const int sign = code >> 7, ex = (code >> 3) & 15, man = code & 7;
    double v;
    if (ex == 15 && man == 7) return NAN;
    if (ex == 0) v = ldexp((double)man / 8.0, -6);
    else v = ldexp(1.0 + (double)man / 8.0, ex - 7);
    return sign ? -v : v;
}

/* Weight rows to E4M3 codes with one scale per row.
 *   scale[r] = max_k |w[r][k]| / 448, computed in float (1 when the row is all zero);
 *   code     = the E4M3 value nearest to the float quotient w / scale, ties to the even
 *              mantissa, magnitudes beyond 448 saturating to 448 (cannot happen here but
 *              is the rule), the sign kept (a negative value that rounds to zero keeps
 *              its sign bit).
 * The nearest value is found by looking at all 127 finite magnitudes: slow and obviously
 * the definition.  Returns 0, or -1 on bad sizes. */
int oracle_quantize_e4m3(const float *w, int64_t rows, int64_t K, uint8_t *codes, float *scale)
{
    if (rows < 0 || K <= 0) return -1;
#pragma omp parallel for schedule(static)              /* rows are independent of each other */
    for (int64_t r = 0; r < rows; ++r) {
        const float *row = w + r * K;
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) { const float a = fabsf(row[k]); if (a > amax) amax = a; }
        const float s = amax > 0.0f ? amax / 448.0f : 1.0f;
        scale[r] = s;
        for (int64_t k = 0; k < K; ++k) {
            const float q = row[k] / s;                  /* float division, as stated */
            const double a = fabs((double)q);
            int best = 0;
            double bd = a;                               /* distance to code 0 */
            for (int c = 1; c <= 0x7e; ++c) {
                const double d = fabs(a - oracle_e4m3_value((uint8_t)c));
                if (d < bd || (d == bd && (c & 1) == 0)) { bd = d; best = c; }
            }
            codes[r * K + k] = (uint8_t)(best | (signbit(q) ? 0x80 : 0));
        }
    }
    return 0;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
