// Fused attention (Sec. 3.3: dequantization, scale computation and the next
// quantization fused into the producing kernel; tensors stay quantized between
// primitives).  Forward = steps 3, 4 and 5 of Fig. 1a in two passes over the
// in-edges without ever writing the fp32 scores E or alpha to memory:
//   pass 1 (k_attn_stats): per (node, head) the maximum of the activated
//          scores and the softmax denominator, plus max(alpha) = max 1/den
//          (the largest term of every softmax row is exp(0) = 1);
//   pass 2 (the SPMM kernel with on-the-fly weights): recomputes alpha per
//          edge from the int8 S_q, D_q (both cache resident), quantizes it,
//          stores the int8 alpha_q for the backward pass and aggregates.
// HBM bytes per edge: pass 1 reads 4 (index); pass 2 reads 4 and writes
// `heads`; the feature-row gathers are as in the plain SPMM.
#include "internal.hip.h"
#include "rowwalk.hip.h"

int tango_spmm_attention_async(const tango_graph *g, int heads, int dim, const int8_t *Sq, const float *sS,
                               const int8_t *Dq, const float *sD, float slope, const float *row_max,
                               const float *row_den, const float *absmax_alpha, int rounding, uint64_t seed,
                               uint64_t stream_id, int8_t *alpha_q, float *s_alpha, float *alpha_dump,
                               const int8_t *X_q, const float *s_X, float *out, float *absmax_out, hipStream_t st);
int tango_validate_spmm_shape(int heads, int dim);
int tango_validate_sddmm_dot_shape(int heads, int dim);
int tango_spmm_async(const tango_graph *g, int direction, int heads, int dim, const int8_t *w_q, const float *s_w,
                     const int8_t *X_q, const float *s_X, float *out, float *absmax_out, hipStream_t st);
int tango_sddmm_dot_async(const tango_graph *g, int heads, int dim, const int8_t *X_dst, const float *s_dst,
                          const int8_t *X_src, const float *s_src, float *out, hipStream_t st);
int tango_attn_bwd_src_async(const tango_graph *g, int heads, int dim, const int8_t *dOut_q, const float *s_dOut,
                             const int8_t *X_q, const float *s_X, const int8_t *Sq, const float *sS, const int8_t *Dq,
                             const float *sD, float slope, const float *row_max, const float *row_den, const double *P,
                             double *dS_acc, float *dS, hipStream_t st);

namespace {

// Online softmax statistics of one row: running maximum m and sum s of exp(E - m).
template <int H>
struct attn_stats_op {
    const int32_t *src;
    const int8_t *Sq, *Dq;
    float sS, sD, slope;
    float *row_max, *row_den;
    float amax;
    template <int GS>
    __device__ void run(int row, int b, int t, int lg)
    {
        float td[H], m[H], s[H];
#pragma unroll
        for (int h = 0; h < H; ++h) {
            td[h] = sD * static_cast<float>(Dq[static_cast<int64_t>(row) * H + h]);
            m[h] = -INFINITY;
            s[h] = 0.0f;
        }
        for (int e = b + lg; e < t; e += GS) {
            const int64_t u = src[e];
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const float ts = sS * static_cast<float>(Sq[u * H + h]);
                const float x = ts + td[h];
                const float ev = x > 0.0f ? x : slope * x;
                if (ev > m[h]) {
                    s[h] = s[h] * expf(m[h] - ev) + 1.0f;
                    m[h] = ev;
                } else {
                    s[h] += expf(ev - m[h]);
                }
            }
        }
#pragma unroll
        for (int h = 0; h < H; ++h) {
#pragma unroll
            for (int o = GS / 2; o > 0; o >>= 1) {
                const float m2 = __shfl_xor(m[h], o, 64), s2 = __shfl_xor(s[h], o, 64);
                const float M = fmaxf(m[h], m2);
                const float f1 = (m[h] == M) ? 1.0f : expf(m[h] - M);
                const float f2 = (m2 == M) ? 1.0f : expf(m2 - M);
                s[h] = s[h] * f1 + s2 * f2;
                m[h] = M;
            }
            if (t > b) {
                if (lg == 0) {
                    row_max[static_cast<int64_t>(row) * H + h] = m[h];
                    row_den[static_cast<int64_t>(row) * H + h] = s[h];
                }
                amax = fmaxf(amax, 1.0f / s[h]);
            } else if (lg == 0) {
                row_max[static_cast<int64_t>(row) * H + h] = 0.0f;
                row_den[static_cast<int64_t>(row) * H + h] = 1.0f;
            }
        }
    }
};

template <int H, int GROUP>
__global__ __launch_bounds__(256) void k_attn_stats(int n, const int32_t *ptr, attn_stats_op<H> op, const float *sS,
                                                    const float *sD, float *absmax_alpha)
{
    op.sS = *sS;
    op.sD = *sD;
    op.amax = 0.0f;
    walk_rows<GROUP>(ptr, n, op);
    const float m = tango_wave_max(op.amax);
    if (threadIdx.x % TANGO_WAVE == 0 && m > 0.0f) tango_atomic_max_nonneg(absmax_alpha, m);
}

// Backward over the in-edges of each destination (steps 4' and 3''): alpha is recomputed from the row statistics,
// P[v][h] = sum dalpha*alpha (fp64), dE = alpha*(dalpha - P), dD[v][h] = sum dE*lrelu'(t).
template <int H>
struct attn_bwd_dst_op {
    const int32_t *src;
    const int8_t *Sq, *Dq;
    float sS, sD, slope;
    const float *row_max, *row_den, *dalpha;
    double *P;
    float *dD;
    template <int GS>
    __device__ void run(int row, int b, int t, int lg)
    {
        float td[H], m[H], den[H];
        double p[H], acc[H];
#pragma unroll
        for (int h = 0; h < H; ++h) {
            td[h] = sD * static_cast<float>(Dq[static_cast<int64_t>(row) * H + h]);
            m[h] = row_max[static_cast<int64_t>(row) * H + h];
            den[h] = row_den[static_cast<int64_t>(row) * H + h];
            p[h] = 0.0;
            acc[h] = 0.0;
        }
        for (int e = b + lg; e < t; e += GS) {
            const int64_t u = src[e];
            float d[H];
            load_h<H>(dalpha + static_cast<int64_t>(e) * H, d);
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const float ts = sS * static_cast<float>(Sq[u * H + h]);
                const float x = ts + td[h];
                const float ev = x > 0.0f ? x : slope * x;
                const float al = expf(ev - m[h]) / den[h];
                p[h] += static_cast<double>(d[h]) * static_cast<double>(al);
            }
        }
#pragma unroll
        for (int h = 0; h < H; ++h) p[h] = group_sum<GS>(p[h]);
        for (int e = b + lg; e < t; e += GS) {
            const int64_t u = src[e];
            float d[H];
            load_h<H>(dalpha + static_cast<int64_t>(e) * H, d);
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const float ts = sS * static_cast<float>(Sq[u * H + h]);
                const float x = ts + td[h];
                const float ev = x > 0.0f ? x : slope * x;
                const float al = expf(ev - m[h]) / den[h];
                const float dE = static_cast<float>(static_cast<double>(al) * (static_cast<double>(d[h]) - p[h]));
                acc[h] += static_cast<double>(dE * (x > 0.0f ? 1.0f : slope));
            }
        }
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const double sacc = group_sum<GS>(acc[h]);
            if (lg == 0) {
                P[static_cast<int64_t>(row) * H + h] = p[h];
                dD[static_cast<int64_t>(row) * H + h] = static_cast<float>(sacc);
            }
        }
    }
};

template <int H, int GROUP>
__global__ __launch_bounds__(256) void k_attn_bwd_dst(int n, const int32_t *ptr, attn_bwd_dst_op<H> op, const float *sS,
                                                      const float *sD)
{
    op.sS = *sS;
    op.sD = *sD;
    walk_rows<GROUP>(ptr, n, op);
}

}  // namespace

int tango_attn_bwd_dst_async(const tango_graph *g, int heads, const int8_t *Sq, const float *sS, const int8_t *Dq,
                             const float *sD, float slope, const float *row_max, const float *row_den,
                             const float *dalpha, double *P, float *dD, hipStream_t st)
{
    const int n = g->n_nodes;
    const int grp = pick_group(n, g->n_edges);
    const unsigned grid = row_grid(n);
#define CALL(HH)                                                                                            \
    {                                                                                                       \
        attn_bwd_dst_op<HH> op{g->in_src, Sq, Dq, 0.f, 0.f, slope, row_max, row_den, dalpha, P, dD};        \
        k_attn_bwd_dst<HH, GROUP><<<grid, 256, 0, st>>>(n, g->in_ptr, op, sS, sD);                          \
    }
    TANGO_DISPATCH_H(heads, grp, CALL)
#undef CALL
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_attn_stats_async(const tango_graph *g, int heads, const int8_t *Sq, const float *sS, const int8_t *Dq,
                           const float *sD, float slope, float *row_max, float *row_den, float *absmax_alpha,
                           hipStream_t st)
{
    const int n = g->n_nodes;
    const int grp = pick_group(n, g->n_edges);
    const unsigned grid = row_grid(n);
    int rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(absmax_alpha), 0u, 1, st);
    if (rc != TANGO_OK) return rc;
#define CALL(HH)                                                                                   \
    {                                                                                              \
        attn_stats_op<HH> op{g->in_src, Sq, Dq, 0.f, 0.f, slope, row_max, row_den, 0.f};           \
        k_attn_stats<HH, GROUP><<<grid, 256, 0, st>>>(n, g->in_ptr, op, sS, sD, absmax_alpha);     \
    }
    TANGO_DISPATCH_H(heads, grp, CALL)
#undef CALL
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

extern "C" {

size_t tango_gat_attention_workspace_bytes(int64_t, int64_t, int) { return 256; }

int tango_gat_attention_fwd(const tango_graph *g, int heads, int dim, const int8_t *S_q, const float *s_S,
                            const int8_t *D_q, const float *s_D, float slope, const int8_t *X_q, const float *s_X,
                            int rounding, uint64_t seed, uint64_t stream_id_alpha, float *row_max, float *row_den,
                            int8_t *alpha_q, float *s_alpha, float *alpha_dump, float *out, float *absmax_out, void *ws,
                            size_t ws_bytes, void *stream)
{
    TANGO_REQUIRE(rounding == TANGO_RN || rounding == TANGO_SR, TANGO_ERR_BAD_ENUM);
    TANGO_REQUIRE(g != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(g->n_nodes > 0 && g->n_edges >= 0 && g->n_edges < (int64_t(1) << 31), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(g->in_ptr && (g->n_edges == 0 || g->in_src), TANGO_ERR_NULL);
    TANGO_REQUIRE(heads_supported(heads), TANGO_ERR_UNSUPPORTED);
    int rc = tango_validate_spmm_shape(heads, dim);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(S_q && s_S && D_q && s_D && X_q && s_X && row_max && row_den && s_alpha && out &&
                      (g->n_edges == 0 || alpha_q),
                  TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(out, 16) && tango_aligned(X_q, 16), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(ws && tango_aligned(ws, 256) && ws_bytes >= 256, TANGO_ERR_WORKSPACE);
    hipStream_t st = tango_stream(stream);
    float *absmax_alpha = static_cast<float *>(ws);
    if (g->n_edges == 0) {  // no edge: the scale of an empty tensor is 1
        rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(s_alpha), 0x3f800000u, 1, st);
        if (rc != TANGO_OK) return rc;
    }
    rc = tango_attn_stats_async(g, heads, S_q, s_S, D_q, s_D, slope, row_max, row_den, absmax_alpha, st);
    if (rc != TANGO_OK) return rc;
    return tango_spmm_attention_async(g, heads, dim, S_q, s_S, D_q, s_D, slope, row_max, row_den, absmax_alpha, rounding,
                                      seed, stream_id_alpha, alpha_q, s_alpha, alpha_dump, X_q, s_X, out, absmax_out, st);
}

size_t tango_gat_attention_bwd_workspace_bytes(int64_t n_nodes, int64_t, int heads)
{
    // P and the dS accumulator: n x heads doubles each
    return 256 + 2 * tango_round_up(static_cast<size_t>(n_nodes) * heads * sizeof(double), 256);
}

int tango_gat_attention_bwd(const tango_graph *g, int heads, int dim, const int8_t *S_q, const float *s_S,
                            const int8_t *D_q, const float *s_D, float slope, const float *row_max, const float *row_den,
                            const int8_t *alpha_q, const float *s_alpha, const int8_t *X_q, const float *s_X,
                            const int8_t *dOut_q, const float *s_dOut, float *dX_agg, float *absmax_dX, float *dalpha,
                            float *dS, float *dD, void *ws, size_t ws_bytes, void *stream)
{
    TANGO_REQUIRE(g != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(g->n_nodes > 0 && g->n_edges >= 0 && g->n_edges < (int64_t(1) << 31), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(g->in_ptr && g->out_ptr && (g->n_edges == 0 || (g->in_src && g->out_dst && g->out_eid)), TANGO_ERR_NULL);
    TANGO_REQUIRE(heads_supported(heads), TANGO_ERR_UNSUPPORTED);
    int rc = tango_validate_sddmm_dot_shape(heads, dim);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(S_q && s_S && D_q && s_D && row_max && row_den && s_alpha && X_q && s_X && dOut_q && s_dOut && dX_agg &&
                      dS && dD && (g->n_edges == 0 || (alpha_q && dalpha)),
                  TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(dX_agg, 16) && tango_aligned(X_q, 16) && tango_aligned(dOut_q, 16) &&
                      tango_aligned(dalpha, 16),
                  TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(ws && tango_aligned(ws, 256) &&
                      ws_bytes >= tango_gat_attention_bwd_workspace_bytes(g->n_nodes, g->n_edges, heads),
                  TANGO_ERR_WORKSPACE);
    hipStream_t st = tango_stream(stream);
    const size_t nh_bytes = tango_round_up(static_cast<size_t>(g->n_nodes) * heads * sizeof(double), 256);
    double *P = reinterpret_cast<double *>(static_cast<char *>(ws) + 256);
    double *dS_acc = reinterpret_cast<double *>(static_cast<char *>(ws) + 256 + nh_bytes);
    // 5': SPMM on the reversed graph with the cached int8 attention
    rc = tango_spmm_async(g, TANGO_OUT, heads, dim, alpha_q, s_alpha, dOut_q, s_dOut, dX_agg, absmax_dX, st);
    if (rc != TANGO_OK) return rc;
    // 5'': dalpha, the only fp32 edge tensor of the backward pass
    rc = tango_sddmm_dot_async(g, heads, dim, dOut_q, s_dOut, X_q, s_X, dalpha, st);
    if (rc != TANGO_OK) return rc;
    // 4' and 3'' over in-edges, then 3' over out-edges
    rc = tango_attn_bwd_dst_async(g, heads, S_q, s_S, D_q, s_D, slope, row_max, row_den, dalpha, P, dD, st);
    if (rc != TANGO_OK) return rc;
    return tango_attn_bwd_src_async(g, heads, dim, dOut_q, s_dOut, X_q, s_X, S_q, s_S, D_q, s_D, slope, row_max, row_den, P,
                                    dS_acc, dS, st);
}

}  // extern "C"
