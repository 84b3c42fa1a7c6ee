/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of the quantization-aware
 * primitives of one GNN training layer (Tango, SC'23): per-tensor symmetric
 * int8 quantization with nearest or stochastic rounding, int8 GEMM with int32
 * accumulation and a dequantize + abs-max step, SDDMM (add and dot), edge
 * softmax forward/backward, SPMM on the graph and on the reversed graph, the
 * edge-to-node sums and the attention-projection steps.
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may use
 * this file.  It shares no code with the GPU library and is never a fallback
 * for it.  Build with:  gcc -O2 -fopenmp -ffp-contract=off -std=c11
 * (no fast-math; fp32 expressions must not be contracted into FMAs because
 * rounding decisions are specified in fp32, one rounding per operation).
 *
 * Conventions: dense tensors row-major; node feature rows hold `heads`
 * blocks of `dim` values (Sec. 2.1, step 1); edge tensors hold `heads` values
 * per edge and are indexed by destination-major edge position; the graph is
 * given destination-major: in-edges of v are in_ptr[v]..in_ptr[v+1]-1 with
 * sources in_src[e].  Every function is pinned by tests that compare it with
 * dense-matrix definitions, closed forms or the paper's printed values; no
 * function here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Counter-based random bits for stochastic rounding.                  */
/* Philox4x32-10 as published by Salmon, Moraes, Dror, Shaw (SC'11):   */
/* the paper only asks for a fast register-resident generator          */
/* (Sec. 3.2, "GPU-accelerated stochastic rounding"); a counter-based  */
/* one makes the bits a pure function of (seed, stream, element).      */
/* ------------------------------------------------------------------ */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * 16 random bits of element i of random stream (seed, stream):
 * one Philox block serves 8 consecutive elements.  key = seed (low, high
 * word), counter = (i/8 low, i/8 high, stream low, stream high); element i
 * takes 32-bit word (i%8)/2 of the block, low half if i is even, high half
 * if i is odd.
 */
uint32_t orc_sr_bits16(uint64_t seed, uint64_t stream, uint64_t i)
{
    uint64_t blk = i >> 3;
    uint32_t ctr[4] = { (uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)stream, (uint32_t)(stream >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    uint32_t w = out[(i & 7) >> 1];
    return (i & 1) ? (w >> 16) : (w & 0xffffu);
}

/* ------------------------------------------------------------------ */
/* Quantization (Sec. 2.3 Eq. 1-2 with Z = 0; Sec. 3.2 Eq. 3).         */
/* ------------------------------------------------------------------ */

/* max_i |x_i| (exact in fp32, order-free). */
float orc_absmax(const float *x, size_t n)
{
    float m = 0.0f;
    for (size_t i = 0; i < n; ++i) {
        float a = fabsf(x[i]);
        if (a > m) m = a;
    }
    return m;
}

/*
 * Symmetric per-tensor scale for B = 8 bits: grid points are s * q with
 * q in [-127, 127] (Fig. 3 gives the range [-127, 127]).  s = absmax / 127,
 * and elements are multiplied by inv = 127 / absmax ("multiply and data type
 * casting", Sec. 3.3).  An all-zero tensor gets s = 1, inv = 0.
 */
void orc_scale_from_absmax(float absmax, float *s, float *inv)
{
    if (absmax > 0.0f) {
        *s = absmax / 127.0f;
        *inv = 127.0f / absmax;
    } else {
        *s = 1.0f;
        *inv = 0.0f;
    }
}

/*
 * q_i = clamp(round(x_i * inv), -127, 127).
 * rounding 0: nearest, ties to even.
 * rounding 1: stochastic (Eq. 3): floor(y) + 1 with probability y - floor(y),
 *             realised as u < frac with u = bits16 * 2^-16.
 * x[0..n) are elements first .. first+n-1 of the tensor (first = 0 for a whole
 * tensor; a window of a large tensor can be checked on its own).
 */
void orc_quantize(const float *x, size_t n, uint64_t first, float absmax, int rounding, uint64_t seed, uint64_t stream,
                  int8_t *q)
{
    float s, inv;
    orc_scale_from_absmax(absmax, &s, &inv);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        float y = x[i] * inv;
        int v;
        if (rounding == 0) {
            v = (int)rintf(y); /* default rounding mode: ties to even */
        } else {
            float f = floorf(y);
            float frac = y - f;
            float u = (float)orc_sr_bits16(seed, stream, first + (uint64_t)i) * (1.0f / 65536.0f);
            v = (int)f + (u < frac ? 1 : 0);
        }
        if (v > 127) v = 127;
        if (v < -127) v = -127;
        q[i] = (int8_t)v;
    }
}

/*
 * B-bit variant of the quantizer (Sec. 3.2 bit-count rule; Sec. 4 "Speed impact
 * for # of quantization bits", INT4): codes in +-(2^(B-1)-1), s = absmax/qmax,
 * inv = qmax/absmax, same rounding rules and the same random bits per element
 * as the 8-bit one.  One code per int8; B = 8 is orc_quantize.
 */
void orc_quantize_bits(const float *x, size_t n, uint64_t first, float absmax, int bits, int rounding, uint64_t seed,
                       uint64_t stream, int8_t *q)
{
    const int qmax = (1 << (bits - 1)) - 1;
    float s = 1.0f, inv = 0.0f;
    if (absmax > 0.0f) {
        s = absmax / (float)qmax;
        inv = (float)qmax / absmax;
    }
    (void)s;
    for (size_t i = 0; i < n; ++i) {
        float y = x[i] * inv;
        int v;
        if (rounding == 0) {
            v = (int)rintf(y);
        } else {
            float f = floorf(y);
            float frac = y - f;
            float u = (float)orc_sr_bits16(seed, stream, first + (uint64_t)i) * (1.0f / 65536.0f);
            v = (int)f + (u < frac ? 1 : 0);
        }
        if (v > qmax) v = qmax;
        if (v < -qmax) v = -qmax;
        q[i] = (int8_t)v;
    }
}

/*
 * Packed 4-bit storage: byte j holds element 2j in its low nibble and element
 * 2j+1 in its high nibble, each as a 4-bit two's-complement number; n even.
 */
void orc_pack_int4(const int8_t *q, size_t n, uint8_t *p)
{
    for (size_t j = 0; j < n / 2; ++j) p[j] = (uint8_t)(((unsigned)q[2 * j] & 0xFu) | (((unsigned)q[2 * j + 1] & 0xFu) << 4));
}

void orc_unpack_int4(const uint8_t *p, size_t n, int8_t *q)
{
    for (size_t j = 0; j < n / 2; ++j) {
        int lo = p[j] & 0xF, hi = p[j] >> 4;
        q[2 * j] = (int8_t)(lo >= 8 ? lo - 16 : lo);
        q[2 * j + 1] = (int8_t)(hi >= 8 ? hi - 16 : hi);
    }
}

/* ------------------------------------------------------------------ */
/* Alternative source of the random bits (Sec. 3.2 "GPU-accelerated      */
/* stochastic rounding": xoshiro256++ with its state kept in registers).  */
/* A generator with state cannot be indexed by element, so the mapping is */
/* fixed instead: 65,536 generators; generator g is seeded by four        */
/* splitmix64 outputs from x0 = seed + stream*0xD1342543DE82EF95 +        */
/* g*0x9E3779B97F4A7C15; one 64-bit output serves the four consecutive    */
/* elements 4v .. 4v+3 (16 bits each, lowest bits first) of group v, and   */
/* group v belongs to generator v % 65536 as its (v / 65536)-th output.    */
/* ------------------------------------------------------------------ */
#define ORC_XO_GENERATORS 65536u

static uint64_t rotl64(uint64_t x, int k) { return (x << k) | (x >> (64 - k)); }

uint64_t orc_splitmix64(uint64_t *x)
{
    uint64_t z = (*x += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* one step of xoshiro256++ (Blackman and Vigna): returns the output, advances s[4] */
uint64_t orc_xoshiro256pp_next(uint64_t s[4])
{
    const uint64_t result = rotl64(s[0] + s[3], 23) + s[0];
    const uint64_t t = s[1] << 17;
    s[2] ^= s[0];
    s[3] ^= s[1];
    s[1] ^= s[2];
    s[0] ^= s[3];
    s[2] ^= t;
    s[3] = rotl64(s[3], 45);
    return result;
}

/* Stochastic-rounding quantizer (Eq. 3) drawing its bits as described above; otherwise orc_quantize. */
void orc_quantize_xoshiro(const float *x, size_t n, float absmax, uint64_t seed, uint64_t stream, int8_t *q)
{
    float s, inv;
    orc_scale_from_absmax(absmax, &s, &inv);
    const uint64_t groups = ((uint64_t)n + 3) / 4;
    for (uint64_t g = 0; g < ORC_XO_GENERATORS && g < groups; ++g) {
        uint64_t x0 = seed + stream * 0xD1342543DE82EF95ull + g * 0x9E3779B97F4A7C15ull;
        uint64_t st[4];
        for (int k = 0; k < 4; ++k) st[k] = orc_splitmix64(&x0);
        for (uint64_t v = g; v < groups; v += ORC_XO_GENERATORS) {
            const uint64_t r = orc_xoshiro256pp_next(st);
            for (int j = 0; j < 4; ++j) {
                const uint64_t i = 4 * v + (uint64_t)j;
                if (i >= n) break;
                const float y = x[i] * inv;
                const float f = floorf(y);
                const float frac = y - f;
                const float u = (float)((r >> (16 * j)) & 0xFFFFu) * (1.0f / 65536.0f);
                int c = (int)f + (u < frac ? 1 : 0);
                if (c > 127) c = 127;
                if (c < -127) c = -127;
                q[i] = (int8_t)c;
            }
        }
    }
}

/* x_i = s * q_i (Eq. 2 with Z = 0). */
void orc_dequantize(const int8_t *q, size_t n, float s, float *x)
{
    for (size_t i = 0; i < n; ++i) x[i] = s * (float)q[i];
}

/* ------------------------------------------------------------------ */
/* Quantization-aware matrix multiplication (Sec. 3.2, Fig. 3).        */
/* ------------------------------------------------------------------ */

/*
 * acc[i][j] = sum_k A(i,k) * B(k,j), A(i,k) = A[i*ars + k*acs],
 * B(k,j) = B[k*brs + j*bcs]; exact (int64), stored as int32.
 * Returns the number of results that do not fit int32 (must be 0).
 */
int64_t orc_igemm(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t ars, int64_t acs, const int8_t *B,
                  int64_t brs, int64_t bcs, int32_t *acc)
{
    int64_t bad = 0;
#pragma omp parallel for schedule(static) reduction(+ : bad)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            int64_t t = 0;
            for (int64_t k = 0; k < K; ++k) t += (int64_t)A[i * ars + k * acs] * (int64_t)B[k * brs + j * bcs];
            if (t > INT32_MAX || t < INT32_MIN) bad += 1;
            acc[i * N + j] = (int32_t)t;
        }
    }
    return bad;
}

/*
 * C = (float)acc * (sa * sb): the two scales are multiplied first (Sec. 3.3,
 * "(s0 * s1) * ..."), then one fp32 multiply per element.  Returns max |C|.
 */
float orc_dequant_i32(const int32_t *acc, size_t n, float sa, float sb, float *C)
{
    float sc = sa * sb;
    float m = 0.0f;
    for (size_t i = 0; i < n; ++i) {
        float c = (float)acc[i] * sc;
        C[i] = c;
        float a = fabsf(c);
        if (a > m) m = a;
    }
    return m;
}

/* ------------------------------------------------------------------ */
/* Step 2: per-head projections S = H' . a_src, D = H' . a_dst.        */
/* out[v][h] = sum_d X[v][h][d] * a[h][d], fp64 sum, one fp32 rounding. */
/* ------------------------------------------------------------------ */
void orc_head_proj(int64_t n, int heads, int dim, const float *X, const float *a, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v)
        for (int h = 0; h < heads; ++h) {
            double t = 0.0;
            for (int d = 0; d < dim; ++d)
                t += (double)X[(size_t)v * heads * dim + (size_t)h * dim + d] * (double)a[h * dim + d];
            out[v * heads + h] = (float)t;
        }
}

/* ------------------------------------------------------------------ */
/* Step 3: SDDMM-add with on-the-fly dequantization + LeakyReLU        */
/* (Sec. 3.3 "SDDMM with on-the-fly dequantization").                  */
/* E[e][h] = lrelu(s_S * S_q[src][h] + s_D * D_q[dst][h]).             */
/* ------------------------------------------------------------------ */
void orc_sddmm_add(int64_t n, const int32_t *in_ptr, const int32_t *in_src, int heads, const int8_t *Sq, float sS,
                   const int8_t *Dq, float sD, float slope, float *E)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t v = 0; v < n; ++v)
        for (int64_t e = in_ptr[v]; e < in_ptr[v + 1]; ++e) {
            int64_t u = in_src[e];
            for (int h = 0; h < heads; ++h) {
                float ts = sS * (float)Sq[u * heads + h];
                float td = sD * (float)Dq[v * heads + h];
                float t = ts + td;
                E[e * heads + h] = t > 0.0f ? t : slope * t;
            }
        }
}

/*
 * Backward of step 3 (steps 3', 3''): grad wrt the pre-activation is
 * dEpost * (t > 0 ? 1 : slope) with t recomputed as above; then
 * dD[v][h] = sum over in-edges of v, dS[u][h] = sum over out-edges of u
 * (fp64 sums, one fp32 rounding).  dEpre may be NULL.
 */
void orc_sddmm_add_bwd(int64_t n, const int32_t *in_ptr, const int32_t *in_src, int heads, const int8_t *Sq,
                       float sS, const int8_t *Dq, float sD, float slope, const float *dEpost, float *dEpre,
                       float *dS, float *dD)
{
    double *accS = (double *)calloc((size_t)n * heads, sizeof(double));
    for (int64_t v = 0; v < n; ++v)
        for (int h = 0; h < heads; ++h) {
            double accD = 0.0;
            for (int64_t e = in_ptr[v]; e < in_ptr[v + 1]; ++e) {
                int64_t u = in_src[e];
                float ts = sS * (float)Sq[u * heads + h];
                float td = sD * (float)Dq[v * heads + h];
                float t = ts + td;
                float g = dEpost[e * heads + h] * (t > 0.0f ? 1.0f : slope);
                if (dEpre) dEpre[e * heads + h] = g;
                accD += (double)g;
                accS[u * heads + h] += (double)g;
            }
            dD[v * heads + h] = (float)accD;
        }
    for (int64_t i = 0; i < n * heads; ++i) dS[i] = (float)accS[i];
    free(accS);
}

/* ------------------------------------------------------------------ */
/* Step 5'': SDDMM-dot on quantized values (Sec. 3.3).                  */
/* out[e][h] = (float)(sum_d Xdst_q[dst][h][d] * Xsrc_q[src][h][d])     */
/*             * (s_dst * s_src).  Returns #int32 overflows (must be 0). */
/* ------------------------------------------------------------------ */
int64_t orc_sddmm_dot(int64_t n, const int32_t *in_ptr, const int32_t *in_src, int heads, int dim,
                      const int8_t *Xdst, float s_dst, const int8_t *Xsrc, float s_src, float *out, int32_t *acc_out)
{
    float sc = s_dst * s_src;
    int64_t bad = 0;
    size_t F = (size_t)heads * dim;
#pragma omp parallel for schedule(dynamic, 256) reduction(+ : bad)
    for (int64_t v = 0; v < n; ++v)
        for (int64_t e = in_ptr[v]; e < in_ptr[v + 1]; ++e) {
            int64_t u = in_src[e];
            for (int h = 0; h < heads; ++h) {
                int64_t t = 0;
                for (int d = 0; d < dim; ++d)
                    t += (int64_t)Xdst[v * F + h * dim + d] * (int64_t)Xsrc[u * F + h * dim + d];
                if (t > INT32_MAX || t < INT32_MIN) bad += 1;
                if (acc_out) acc_out[e * heads + h] = (int32_t)t;
                out[e * heads + h] = (float)(int32_t)t * sc;
            }
        }
    return bad;
}

/* ------------------------------------------------------------------ */
/* Step 4: edge softmax over the in-edges of each node, per head, in   */
/* full precision (Sec. 3.2, "Full precision for the layer before      */
/* Softmax").  The row maximum is subtracted first (same value         */
/* mathematically); sums and exp in fp64, one fp32 rounding.            */
/* ------------------------------------------------------------------ */
void orc_edge_softmax(int64_t n, const int32_t *in_ptr, int heads, const float *E, float *alpha)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t v = 0; v < n; ++v)
        for (int h = 0; h < heads; ++h) {
            int64_t b = in_ptr[v], t = in_ptr[v + 1];
            if (b == t) continue;
            double m = -INFINITY;
            for (int64_t e = b; e < t; ++e)
                if ((double)E[e * heads + h] > m) m = (double)E[e * heads + h];
            double den = 0.0;
            for (int64_t e = b; e < t; ++e) den += exp((double)E[e * heads + h] - m);
            for (int64_t e = b; e < t; ++e) alpha[e * heads + h] = (float)(exp((double)E[e * heads + h] - m) / den);
        }
}

/*
 * Step 4': P[v][h] = sum_{e->v} dalpha * alpha; dE = alpha * (dalpha - P).
 */
void orc_edge_softmax_bwd(int64_t n, const int32_t *in_ptr, int heads, const float *alpha, const float *dalpha,
                          float *dE)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t v = 0; v < n; ++v)
        for (int h = 0; h < heads; ++h) {
            double P = 0.0;
            for (int64_t e = in_ptr[v]; e < in_ptr[v + 1]; ++e)
                P += (double)dalpha[e * heads + h] * (double)alpha[e * heads + h];
            for (int64_t e = in_ptr[v]; e < in_ptr[v + 1]; ++e)
                dE[e * heads + h] = (float)((double)alpha[e * heads + h] * ((double)dalpha[e * heads + h] - P));
        }
}

/* ------------------------------------------------------------------ */
/* Step 5: quantized SPMM, H_out = (G (.) w) . X over in-edges.         */
/* acc[v][h][d] = sum_{e=(u->v)} w_q[e][h] * X_q[u][h][d] exactly,      */
/* out = (float)acc * (s_w * s_X).  Returns #int32 overflows (must be   */
/* 0); *absmax gets max |out|.  acc_out (int32, n x F) may be NULL.      */
/* ------------------------------------------------------------------ */
int64_t orc_spmm_in(int64_t n, const int32_t *in_ptr, const int32_t *in_src, int heads, int dim, const int8_t *wq,
                    float sw, const int8_t *Xq, float sX, float *out, float *absmax, int32_t *acc_out)
{
    float sc = sw * sX;
    size_t F = (size_t)heads * dim;
    int64_t bad = 0;
    float gm = 0.0f;
#pragma omp parallel reduction(+ : bad)
    {
        int64_t *acc = (int64_t *)malloc(F * sizeof(int64_t));
        float lm = 0.0f;
#pragma omp for schedule(dynamic, 64)
        for (int64_t v = 0; v < n; ++v) {
            memset(acc, 0, F * sizeof(int64_t));
            for (int64_t e = in_ptr[v]; e < in_ptr[v + 1]; ++e) {
                int64_t u = in_src[e];
                for (int h = 0; h < heads; ++h) {
                    int64_t w = wq[e * heads + h];
                    for (int d = 0; d < dim; ++d) acc[h * dim + d] += w * (int64_t)Xq[u * F + h * dim + d];
                }
            }
            for (size_t c = 0; c < F; ++c) {
                if (acc[c] > INT32_MAX || acc[c] < INT32_MIN) bad += 1;
                if (acc_out) acc_out[v * F + c] = (int32_t)acc[c];
                float o = (float)(int32_t)acc[c] * sc;
                out[v * F + c] = o;
                if (fabsf(o) > lm) lm = fabsf(o);
            }
        }
#pragma omp critical
        if (lm > gm) gm = lm;
        free(acc);
    }
    if (absmax) *absmax = gm;
    return bad;
}

/*
 * Step 5': SPMM on the reversed graph, dX = (G^T (.) w) . Y:
 * acc[u][h][d] = sum_{e=(u->v)} w_q[e][h] * Y_q[v][h][d], written as a
 * scatter along the same destination-major edge list (so it does not use
 * the source-major index arrays).  Threads split the feature columns.
 */
int64_t orc_spmm_rev(int64_t n, const int32_t *in_ptr, const int32_t *in_src, int heads, int dim, const int8_t *wq,
                     float sw, const int8_t *Yq, float sY, float *out, float *absmax, int32_t *acc_out)
{
    float sc = sw * sY;
    size_t F = (size_t)heads * dim;
    int64_t *acc = (int64_t *)calloc((size_t)n * F, sizeof(int64_t));
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < (int64_t)F; ++c) {
        int h = (int)(c / dim);
        for (int64_t v = 0; v < n; ++v)
            for (int64_t e = in_ptr[v]; e < in_ptr[v + 1]; ++e) {
                int64_t u = in_src[e];
                acc[u * F + c] += (int64_t)wq[e * heads + h] * (int64_t)Yq[v * F + c];
            }
    }
    int64_t bad = 0;
    float m = 0.0f;
    for (size_t i = 0; i < (size_t)n * F; ++i) {
        if (acc[i] > INT32_MAX || acc[i] < INT32_MIN) bad += 1;
        if (acc_out) acc_out[i] = (int32_t)acc[i];
        float o = (float)(int32_t)acc[i] * sc;
        out[i] = o;
        if (fabsf(o) > m) m = fabsf(o);
    }
    free(acc);
    if (absmax) *absmax = m;
    return bad;
}

/* ------------------------------------------------------------------ */
/* Step 2': backward of the per-head projections.                       */
/* dX_att[v][h][d] = dS[v][h]*a_src[h][d] + dD[v][h]*a_dst[h][d]        */
/*   (two fp32 products, one fp32 sum, no contraction);                 */
/* dX[v][h][d]     = dX_agg + dX_att  (one more fp32 sum);              */
/* da_src[h][d]    = sum_v dS[v][h] * (sX * X_q[v][h][d]), fp64 sum;    */
/* da_dst likewise with dD.  Returns max |dX|.                          */
/* ------------------------------------------------------------------ */
float orc_head_proj_bwd(int64_t n, int heads, int dim, const float *dS, const float *dD, const float *a_src,
                        const float *a_dst, const int8_t *Xq, float sX, const float *dX_agg, float *dX,
                        float *da_src, float *da_dst)
{
    size_t F = (size_t)heads * dim;
    float m = 0.0f;
    double *as = (double *)calloc(F, sizeof(double));
    double *ad = (double *)calloc(F, sizeof(double));
    for (int64_t v = 0; v < n; ++v)
        for (int h = 0; h < heads; ++h)
            for (int d = 0; d < dim; ++d) {
                size_t c = (size_t)h * dim + d;
                float p0 = dS[v * heads + h] * a_src[c];
                float p1 = dD[v * heads + h] * a_dst[c];
                float att = p0 + p1;
                float t = dX_agg[v * F + c] + att;
                dX[v * F + c] = t;
                if (fabsf(t) > m) m = fabsf(t);
                float x = sX * (float)Xq[v * F + c];
                as[c] += (double)dS[v * heads + h] * (double)x;
                ad[c] += (double)dD[v * heads + h] * (double)x;
            }
    for (size_t c = 0; c < F; ++c) {
        da_src[c] = (float)as[c];
        da_dst[c] = (float)ad[c];
    }
    free(as);
    free(ad);
    return m;
}

/* ------------------------------------------------------------------ */
/* Full-precision twins (the non-quantized primitives the quantized    */
/* ones are compared with, Sec. 2.1 steps 5 and 5''): same products in  */
/* fp32 storage, sums in fp64, one fp32 rounding.                       */
/* ------------------------------------------------------------------ */
void orc_spmm_f32(int64_t n, const int32_t *in_ptr, const int32_t *in_src, int heads, int dim, const float *w,
                  const float *X, int reverse, float *out)
{
    size_t F = (size_t)heads * dim;
    double *acc = (double *)calloc((size_t)n * F, sizeof(double));
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < (int64_t)F; ++c) {
        int h = (int)(c / dim);
        for (int64_t v = 0; v < n; ++v)
            for (int64_t e = in_ptr[v]; e < in_ptr[v + 1]; ++e) {
                int64_t u = in_src[e];
                if (reverse)
                    acc[u * F + c] += (double)w[e * heads + h] * (double)X[v * F + c];
                else
                    acc[v * F + c] += (double)w[e * heads + h] * (double)X[u * F + c];
            }
    }
    for (size_t i = 0; i < (size_t)n * F; ++i) out[i] = (float)acc[i];
    free(acc);
}

void orc_sddmm_dot_f32(int64_t n, const int32_t *in_ptr, const int32_t *in_src, int heads, int dim, const float *Xdst,
                       const float *Xsrc, float *out)
{
    size_t F = (size_t)heads * dim;
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t v = 0; v < n; ++v)
        for (int64_t e = in_ptr[v]; e < in_ptr[v + 1]; ++e) {
            int64_t u = in_src[e];
            for (int h = 0; h < heads; ++h) {
                double t = 0.0;
                for (int d = 0; d < dim; ++d) t += (double)Xdst[v * F + h * dim + d] * (double)Xsrc[u * F + h * dim + d];
                out[e * heads + h] = (float)t;
            }
        }
}

/* ------------------------------------------------------------------ */
/* Quantization-error metric and bit-count rule (Sec. 3.2, Eq. 4).      */
/* Error_X = mean_i | (X_i - X_i,Quant) / (X_i + X_i,Quant + eps) |,     */
/* eps = 0.0005, X_i,Quant the grid point s*q_i of a B-bit symmetric     */
/* quantizer (codes in +-(2^(B-1)-1), same scale/rounding rules as the   */
/* 8-bit one).  Terms and their sum in fp64.                              */
/* ------------------------------------------------------------------ */
double orc_error_x(const float *x, size_t n, int bits, float absmax, int rounding, uint64_t seed, uint64_t stream)
{
    const float qmax = (float)((1 << (bits - 1)) - 1);
    float s = 1.0f, inv = 0.0f;
    if (absmax > 0.0f) {
        s = absmax / qmax;
        inv = qmax / absmax;
    }
    double sum = 0.0;
    for (size_t i = 0; i < n; ++i) {
        float y = x[i] * inv;
        float v;
        if (rounding == 0) {
            v = rintf(y);
        } else {
            float f = floorf(y);
            float frac = y - f;
            float u = (float)orc_sr_bits16(seed, stream, (uint64_t)i) * (1.0f / 65536.0f);
            v = f + (u < frac ? 1.0f : 0.0f);
        }
        if (v > qmax) v = qmax;
        if (v < -qmax) v = -qmax;
        float xq = s * v;
        sum += fabs(((double)x[i] - (double)xq) / ((double)x[i] + (double)xq + 0.0005));
    }
    return n ? sum / (double)n : 0.0;
}
