// Streaming edge primitives in full precision: SDDMM-add with on-the-fly
// dequantization + LeakyReLU (Sec. 2.1 step 3, Sec. 3.3), its backward with the
// edge-to-node sums (steps 3', 3''; Sec. 3.3 Fig. 5), edge softmax forward and
// backward (steps 4, 4'; Sec. 3.2 keeps them in fp32).
//
// All of them stream the destination-major edge arrays once or a few times
// and are bound by HBM bandwidth.  Rows (nodes) are handed out in blocks of 64
// consecutive rows per wavefront; short rows are processed by groups of GROUP
// lanes (GROUP ~ the mean degree), rows longer than 16*GROUP by the whole
// wave, one lane per edge with all heads of that edge.
#include "internal.hip.h"
#include "rowwalk.hip.h"

namespace {

// ------------------------------------------------------------------ SDDMM-add
template <int H>
struct sddmm_add_op {
    const int32_t *src;
    const int8_t *Sq, *Dq;
    float sS, sD, slope;
    float *E;
    template <class Team>
    __device__ void run(int row, int b, int t, Team tm)
    {
        float td[H];
#pragma unroll
        for (int h = 0; h < H; ++h) td[h] = sD * static_cast<float>(Dq[static_cast<int64_t>(row) * H + h]);
        for (int e = b + tm.rank; e < t; e += tm.size()) {
            const int64_t u = src[e];
            float v[H];
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const float ts = sS * static_cast<float>(Sq[u * H + h]);
                const float x = ts + td[h];
                v[h] = x > 0.0f ? x : slope * x;
            }
            store_h<H>(E + static_cast<int64_t>(e) * H, v);
        }
    }
};

template <int H, int GROUP>
__global__ __launch_bounds__(256) void k_sddmm_add(int n, const int32_t *ptr, sddmm_add_op<H> op, const float *sS,
                                                   const float *sD)
{
    op.sS = *sS;
    op.sD = *sD;
    walk_rows<GROUP>(ptr, n, op);
}

// dD[v][h] = sum over in-edges of dE*lrelu'(t); optional dE_pre.
template <int H>
struct sddmm_add_bwd_dst_op {
    const int32_t *src;
    const int8_t *Sq, *Dq;
    float sS, sD, slope;
    const float *dE;
    float *dEpre, *dD;
    template <class Team>
    __device__ void run(int row, int b, int t, Team tm)
    {
        float td[H];
        double acc[H];
#pragma unroll
        for (int h = 0; h < H; ++h) {
            td[h] = sD * static_cast<float>(Dq[static_cast<int64_t>(row) * H + h]);
            acc[h] = 0.0;
        }
        for (int e = b + tm.rank; e < t; e += tm.size()) {
            const int64_t u = src[e];
            float g[H];
            load_h<H>(dE + static_cast<int64_t>(e) * H, g);
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const float ts = sS * static_cast<float>(Sq[u * H + h]);
                const float x = ts + td[h];
                g[h] = g[h] * (x > 0.0f ? 1.0f : slope);
                acc[h] += static_cast<double>(g[h]);
            }
            if (dEpre) store_h<H>(dEpre + static_cast<int64_t>(e) * H, g);
        }
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const double s = tm.sum(acc[h]);
            if (tm.rank == 0) dD[static_cast<int64_t>(row) * H + h] = static_cast<float>(s);
        }
    }
};

template <int H, int GROUP>
__global__ __launch_bounds__(256) void k_sddmm_add_bwd_dst(int n, const int32_t *ptr, sddmm_add_bwd_dst_op<H> op,
                                                           const float *sS, const float *sD)
{
    op.sS = *sS;
    op.sD = *sD;
    walk_rows<GROUP>(ptr, n, op);
}

// dS[u][h] = sum over out-edges of dE[eid]*lrelu'(t), t recomputed from S_q[u], D_q[dst].
template <int H>
struct sddmm_add_bwd_src_op {
    const int32_t *dst, *eid;
    const int8_t *Sq, *Dq;
    float sS, sD, slope;
    const float *dE;
    float *dS;
    template <class Team>
    __device__ void run(int row, int b, int t, Team tm)
    {
        float ts[H];
        double acc[H];
#pragma unroll
        for (int h = 0; h < H; ++h) {
            ts[h] = sS * static_cast<float>(Sq[static_cast<int64_t>(row) * H + h]);
            acc[h] = 0.0;
        }
        for (int j = b + tm.rank; j < t; j += tm.size()) {
            const int64_t v = dst[j];
            const int64_t e = eid[j];
            float g[H];
            load_h<H>(dE + e * H, g);
#pragma unroll
            for (int h = 0; h < H; ++h) {
                const float tdv = sD * static_cast<float>(Dq[v * H + h]);
                const float x = ts[h] + tdv;
                acc[h] += static_cast<double>(g[h] * (x > 0.0f ? 1.0f : slope));
            }
        }
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const double s = tm.sum(acc[h]);
            if (tm.rank == 0) dS[static_cast<int64_t>(row) * H + h] = static_cast<float>(s);
        }
    }
};

template <int H, int GROUP>
__global__ __launch_bounds__(256) void k_sddmm_add_bwd_src(int n, const int32_t *ptr, sddmm_add_bwd_src_op<H> op,
                                                           const float *sS, const float *sD)
{
    op.sS = *sS;
    op.sD = *sD;
    walk_rows<GROUP>(ptr, n, op);
}

// ------------------------------------------------------------------ edge softmax
template <int H>
struct softmax_op {
    const float *E;
    float *alpha;
    float amax;
    template <class Team>
    __device__ void run(int /*row*/, int b, int t, Team tm)
    {
        float m[H], s[H];
#pragma unroll
        for (int h = 0; h < H; ++h) {
            m[h] = -INFINITY;
            s[h] = 0.0f;
        }
        for (int e = b + tm.rank; e < t; e += tm.size()) {
            float v[H];
            load_h<H>(E + static_cast<int64_t>(e) * H, v);
#pragma unroll
            for (int h = 0; h < H; ++h) m[h] = fmaxf(m[h], v[h]);
        }
#pragma unroll
        for (int h = 0; h < H; ++h) m[h] = tm.max(m[h]);
        for (int e = b + tm.rank; e < t; e += tm.size()) {
            float v[H];
            load_h<H>(E + static_cast<int64_t>(e) * H, v);
#pragma unroll
            for (int h = 0; h < H; ++h) s[h] += expf(v[h] - m[h]);
        }
#pragma unroll
        for (int h = 0; h < H; ++h) s[h] = tm.sum(s[h]);
        for (int e = b + tm.rank; e < t; e += tm.size()) {
            float v[H];
            load_h<H>(E + static_cast<int64_t>(e) * H, v);
#pragma unroll
            for (int h = 0; h < H; ++h) {
                v[h] = expf(v[h] - m[h]) / s[h];
                amax = fmaxf(amax, v[h]);
            }
            store_h<H>(alpha + static_cast<int64_t>(e) * H, v);
        }
    }
};

template <int H, int GROUP>
__global__ __launch_bounds__(256) void k_edge_softmax(int n, const int32_t *ptr, softmax_op<H> op, float *absmax)
{
    op.amax = 0.0f;
    walk_rows<GROUP>(ptr, n, op);
    if (absmax) {
        const float m = tango_wave_max(op.amax);
        if (threadIdx.x % TANGO_WAVE == 0 && m > 0.0f) tango_atomic_max_nonneg(absmax, m);
    }
}

template <int H>
struct softmax_bwd_op {
    const float *alpha, *dalpha;
    float *dE;
    template <class Team>
    __device__ void run(int /*row*/, int b, int t, Team tm)
    {
        double P[H];
#pragma unroll
        for (int h = 0; h < H; ++h) P[h] = 0.0;
        for (int e = b + tm.rank; e < t; e += tm.size()) {
            float a[H], d[H];
            load_h<H>(alpha + static_cast<int64_t>(e) * H, a);
            load_h<H>(dalpha + static_cast<int64_t>(e) * H, d);
#pragma unroll
            for (int h = 0; h < H; ++h) P[h] += static_cast<double>(d[h]) * static_cast<double>(a[h]);
        }
#pragma unroll
        for (int h = 0; h < H; ++h) P[h] = tm.sum(P[h]);
        for (int e = b + tm.rank; e < t; e += tm.size()) {
            float a[H], d[H], o[H];
            load_h<H>(alpha + static_cast<int64_t>(e) * H, a);
            load_h<H>(dalpha + static_cast<int64_t>(e) * H, d);
#pragma unroll
            for (int h = 0; h < H; ++h)
                o[h] = static_cast<float>(static_cast<double>(a[h]) * (static_cast<double>(d[h]) - P[h]));
            store_h<H>(dE + static_cast<int64_t>(e) * H, o);
        }
    }
};

template <int H, int GROUP>
__global__ __launch_bounds__(256) void k_edge_softmax_bwd(int n, const int32_t *ptr, softmax_bwd_op<H> op)
{
    walk_rows<GROUP>(ptr, n, op);
}

}  // namespace

int tango_sddmm_add_async(const tango_graph *g, int heads, const int8_t *Sq, const float *sS, const int8_t *Dq,
                          const float *sD, float slope, float *E, hipStream_t st)
{
    const int n = g->n_nodes;
    const int grp = pick_group(n, g->n_edges);
    const unsigned grid = row_grid(n, grp);
#define CALL(HH)                                                                        \
    {                                                                                   \
        sddmm_add_op<HH> op{g->in_src, Sq, Dq, 0.f, 0.f, slope, E};                     \
        k_sddmm_add<HH, GROUP><<<grid, 256, 0, st>>>(n, g->in_ptr, op, sS, sD);         \
    }
    TANGO_DISPATCH_H(heads, grp, CALL)
#undef CALL
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_sddmm_add_bwd_async(const tango_graph *g, int heads, const int8_t *Sq, const float *sS, const int8_t *Dq,
                              const float *sD, float slope, const float *dE, float *dEpre, float *dS, float *dD,
                              hipStream_t st)
{
    const int n = g->n_nodes;
    const int grp = pick_group(n, g->n_edges);
    const unsigned grid = row_grid(n, grp);
    if (dD || dEpre) {
#define CALL(HH)                                                                                \
    {                                                                                           \
        sddmm_add_bwd_dst_op<HH> op{g->in_src, Sq, Dq, 0.f, 0.f, slope, dE, dEpre, dD};         \
        k_sddmm_add_bwd_dst<HH, GROUP><<<grid, 256, 0, st>>>(n, g->in_ptr, op, sS, sD);         \
    }
        TANGO_DISPATCH_H(heads, grp, CALL)
#undef CALL
        TANGO_LAUNCH_CHECK();
    }
    if (dS) {
#define CALL(HH)                                                                                \
    {                                                                                           \
        sddmm_add_bwd_src_op<HH> op{g->out_dst, g->out_eid, Sq, Dq, 0.f, 0.f, slope, dE, dS};   \
        k_sddmm_add_bwd_src<HH, GROUP><<<grid, 256, 0, st>>>(n, g->out_ptr, op, sS, sD);        \
    }
        TANGO_DISPATCH_H(heads, grp, CALL)
#undef CALL
        TANGO_LAUNCH_CHECK();
    }
    return TANGO_OK;
}

int tango_edge_softmax_async(const tango_graph *g, int heads, const float *E, float *alpha, float *absmax,
                             hipStream_t st)
{
    const int n = g->n_nodes;
    const int grp = pick_group(n, g->n_edges);
    const unsigned grid = row_grid(n, grp);
    if (absmax) {
        int rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(absmax), 0u, 1, st);
        if (rc != TANGO_OK) return rc;
    }
#define CALL(HH)                                                                    \
    {                                                                               \
        softmax_op<HH> op{E, alpha, 0.f};                                           \
        k_edge_softmax<HH, GROUP><<<grid, 256, 0, st>>>(n, g->in_ptr, op, absmax);  \
    }
    TANGO_DISPATCH_H(heads, grp, CALL)
#undef CALL
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_edge_softmax_bwd_async(const tango_graph *g, int heads, const float *alpha, const float *dalpha, float *dE,
                                 hipStream_t st)
{
    const int n = g->n_nodes;
    const int grp = pick_group(n, g->n_edges);
    const unsigned grid = row_grid(n, grp);
#define CALL(HH)                                                                \
    {                                                                           \
        softmax_bwd_op<HH> op{alpha, dalpha, dE};                               \
        k_edge_softmax_bwd<HH, GROUP><<<grid, 256, 0, st>>>(n, g->in_ptr, op);  \
    }
    TANGO_DISPATCH_H(heads, grp, CALL)
#undef CALL
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_sddmm_dot_async(const tango_graph *g, int heads, int dim, const int8_t *X_dst, const float *s_dst,
                          const int8_t *X_src, const float *s_src, float *out, hipStream_t st);
int tango_validate_sddmm_dot_shape(int heads, int dim);

namespace {
int validate_in_graph(const tango_graph *g)
{
    TANGO_REQUIRE(g != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(g->n_nodes > 0 && g->n_edges >= 0 && g->n_edges < (int64_t(1) << 31), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(g->in_ptr && (g->n_edges == 0 || g->in_src), TANGO_ERR_NULL);
    return TANGO_OK;
}
}  // namespace

extern "C" {

int tango_qsddmm(const tango_graph *g, int op, int heads, int dim, const int8_t *X_src, const float *s_src,
                 const int8_t *X_dst, const float *s_dst, float slope, float *E, void *stream)
{
    TANGO_REQUIRE(op == TANGO_SDDMM_ADD_LEAKYRELU || op == TANGO_SDDMM_DOT, TANGO_ERR_BAD_ENUM);
    int rc = validate_in_graph(g);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(X_src && X_dst && s_src && s_dst && (g->n_edges == 0 || E), TANGO_ERR_NULL);
    if (op == TANGO_SDDMM_ADD_LEAKYRELU) {
        TANGO_REQUIRE(dim == 1, TANGO_ERR_BAD_SHAPE);
        TANGO_REQUIRE(heads_supported(heads), TANGO_ERR_UNSUPPORTED);
        TANGO_REQUIRE(tango_aligned(E, 16), TANGO_ERR_BAD_SHAPE);
        return tango_sddmm_add_async(g, heads, X_src, s_src, X_dst, s_dst, slope, E, tango_stream(stream));
    }
    rc = tango_validate_sddmm_dot_shape(heads, dim);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(tango_aligned(X_src, 16) && tango_aligned(X_dst, 16), TANGO_ERR_BAD_SHAPE);
    return tango_sddmm_dot_async(g, heads, dim, X_dst, s_dst, X_src, s_src, E, tango_stream(stream));
}

int tango_qsddmm_bwd(const tango_graph *g, int heads, const int8_t *X_src, const float *s_src, const int8_t *X_dst,
                     const float *s_dst, float slope, const float *dE, float *dE_pre, float *dS, float *dD, void *stream)
{
    int rc = validate_in_graph(g);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(heads_supported(heads), TANGO_ERR_UNSUPPORTED);
    TANGO_REQUIRE(X_src && X_dst && s_src && s_dst && (g->n_edges == 0 || dE), TANGO_ERR_NULL);
    if (dS) TANGO_REQUIRE(g->out_ptr && (g->n_edges == 0 || (g->out_dst && g->out_eid)), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(dE, 16) && tango_aligned(dE_pre, 16), TANGO_ERR_BAD_SHAPE);
    return tango_sddmm_add_bwd_async(g, heads, X_src, s_src, X_dst, s_dst, slope, dE, dE_pre, dS, dD,
                                     tango_stream(stream));
}

int tango_edge_softmax(const tango_graph *g, int heads, const float *E, float *alpha, float *absmax_alpha, void *stream)
{
    int rc = validate_in_graph(g);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(heads_supported(heads), TANGO_ERR_UNSUPPORTED);
    TANGO_REQUIRE(g->n_edges == 0 || (E && alpha), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(E, 16) && tango_aligned(alpha, 16), TANGO_ERR_BAD_SHAPE);
    return tango_edge_softmax_async(g, heads, E, alpha, absmax_alpha, tango_stream(stream));
}

int tango_edge_softmax_bwd(const tango_graph *g, int heads, const float *alpha, const float *dalpha, float *dE,
                           void *stream)
{
    int rc = validate_in_graph(g);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(heads_supported(heads), TANGO_ERR_UNSUPPORTED);
    TANGO_REQUIRE(g->n_edges == 0 || (alpha && dalpha && dE), TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(alpha, 16) && tango_aligned(dalpha, 16) && tango_aligned(dE, 16), TANGO_ERR_BAD_SHAPE);
    return tango_edge_softmax_bwd_async(g, heads, alpha, dalpha, dE, tango_stream(stream));
}

}  // extern "C"
