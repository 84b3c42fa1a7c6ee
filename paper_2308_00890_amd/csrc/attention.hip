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
#include "attn_math.hip.h"
#include "rowwalk.hip.h"

int tango_spmm_attention_async(const tango_graph *g, int direction, int heads, int dim, const int8_t *Sq,
                               const float *sS, const int8_t *Dq, const float *sD, float slope, const float *row_lse,
                               const float *absmax_alpha, int rounding, uint64_t seed, uint64_t stream_id,
                               int8_t *alpha_q, float *s_alpha, float *alpha_dump, const int8_t *X_q, const float *s_X,
                               float *out, float *absmax_out, int relu_out, uint16_t *relu_bits, const int8_t *src_codes,
                               hipStream_t st, bool out_prezeroed = false);
int tango_spmm_attention_rev_ds_async(const tango_graph *g, int heads, int dim, const int8_t *Sq, const float *sS,
                                      const int8_t *Dq, const float *sD, float slope, const float *row_lse,
                                      const float *absmax_alpha, int rounding, uint64_t seed, uint64_t stream_id,
                                      const float *s_alpha, const int8_t *dOut_q, const float *s_dOut, const int8_t *X_q,
                                      const float *s_X, const void *rec, double *dS_acc, float *out,
                                      float *absmax_out, float *dS, bool dS_acc_zeroed, hipStream_t st, bool out_prezeroed = false);
int tango_attn_bwd_dst_fused_async(const tango_graph *g, int heads, int dim, const int8_t *dOut_q, const float *s_dOut,
                                   const int8_t *X_q, const float *s_X, const int8_t *Sq, const float *sS, const int8_t *Dq,
                                   const float *sD, float slope, const float *row_lse, double *stats, void *rec,
                                   float *dD, const int8_t *src_codes, double *also_zero, bool prezeroed, hipStream_t st);
int tango_validate_spmm_shape(int heads, int dim);
int tango_validate_sddmm_dot_shape(int heads, int dim);
int tango_spmm_async(const tango_graph *g, int direction, int heads, int dim, const int8_t *w_q, const float *s_w,
                     const int8_t *X_q, const float *s_X, float *out, float *absmax_out, hipStream_t st);
int tango_sddmm_dot_async(const tango_graph *g, int heads, int dim, const int8_t *X_dst, const float *s_dst,
                          const int8_t *X_src, const float *s_src, float *out, hipStream_t st);
int tango_attn_bwd_src_async(const tango_graph *g, int heads, int dim, const int8_t *dOut_q, const float *s_dOut,
                             const int8_t *X_q, const float *s_X, const int8_t *Sq, const float *sS, const int8_t *Dq,
                             const float *sD, float slope, const void *rec, double *dS_acc, float *dS,
                             hipStream_t st);

namespace {

// Online softmax statistics of one row: running maximum m and sum s of exp(E - m).
template <int H>
struct attn_stats_op {
    const int32_t *src;
    const int8_t *Sq, *Dq;
    float sS, sD, slope;
    float *row_lse;
    float amax;
    int8_t *src_codes;  // optional: S_q of every edge's source, in edge order (written here, read by the later walks)
    template <class Team>
    __device__ void run(int row, int b, int t, Team tm)
    {
        float td[H], m[H], s[H];
        int dq[H];
        tango_load_heads<H>(Dq, row, dq);
#pragma unroll
        for (int h = 0; h < H; ++h) {
            td[h] = sD * static_cast<float>(dq[h]);
            m[h] = -INFINITY;
            s[h] = 0.0f;
        }
        // four edges per lane and iteration: the four index loads, then the four gathers, are issued back to back, and
        // the running maximum is raised once per group (one rescaling exponential per four edges instead of one each)
        constexpr int UE = 4;
        int e = b + tm.rank;
        for (; e + (UE - 1) * tm.size() < t; e += UE * tm.size()) {
            int nb[UE];
#pragma unroll
            for (int u = 0; u < UE; ++u) nb[u] = src[e + u * tm.size()];
            int sq[UE][H];
#pragma unroll
            for (int u = 0; u < UE; ++u) tango_load_heads<H>(Sq, nb[u], sq[u]);
            if (src_codes) {
#pragma unroll
                for (int u = 0; u < UE; ++u) tango_store_heads<H>(src_codes, e + u * tm.size(), sq[u]);
            }
#pragma unroll
            for (int h = 0; h < H; ++h) {
                float ev[UE];
                float mx = m[h];
#pragma unroll
                for (int u = 0; u < UE; ++u) {
                    bool pos;
                    ev[u] = tango_attn_score(sS * static_cast<float>(sq[u][h]), td[h], slope, pos);
                    mx = fmaxf(mx, ev[u]);
                }
                float acc = (mx > m[h]) ? s[h] * tango_attn_exp(m[h] - mx) : s[h];
#pragma unroll
                for (int u = 0; u < UE; ++u) acc += tango_attn_exp(ev[u] - mx);
                s[h] = acc;
                m[h] = mx;
            }
        }
        for (; e < t; e += tm.size()) {
            int sq[H];
            tango_load_heads<H>(Sq, src[e], sq);
            if (src_codes) tango_store_heads<H>(src_codes, e, sq);
#pragma unroll
            for (int h = 0; h < H; ++h) {
                bool pos;
                const float ev = tango_attn_score(sS * static_cast<float>(sq[h]), td[h], slope, pos);
                if (ev > m[h]) {
                    s[h] = s[h] * tango_attn_exp(m[h] - ev) + 1.0f;
                    m[h] = ev;
                } else {
                    s[h] += tango_attn_exp(ev - m[h]);
                }
            }
        }
#pragma unroll
        for (int h = 0; h < H; ++h) {
            tm.merge_ms(m[h], s[h]);
            if (t > b) {
                const float lse = m[h] + logf(s[h]);
                if (tm.rank == 0) row_lse[static_cast<int64_t>(row) * H + h] = lse;
                amax = fmaxf(amax, tango_attn_alpha(m[h], lse));  // the largest alpha of the row: its maximum score
            } else if (tm.rank == 0) {
                row_lse[static_cast<int64_t>(row) * H + h] = 0.0f;
            }
        }
    }
};

// The workgroups below huge_blocks take the rows longer than HUGE_ROW, a whole workgroup per row; the others walk the
// remaining rows with a group of lanes per row.  One launch: the hub rows no longer wait for the short ones.
template <int H, int GROUP>
__global__ __launch_bounds__(256) void k_attn_stats(int n, const int32_t *ptr, attn_stats_op<H> op, const float *sS,
                                                    const float *sD, float *absmax_alpha, int huge_blocks, int rows_per_wave)
{
    __shared__ double scratch[2 * 256 / 64];
    __shared__ int list[256 + 1];
    op.sS = *sS;
    op.sD = *sD;
    op.amax = 0.0f;
    if (static_cast<int>(blockIdx.x) < huge_blocks)
        walk_huge_rows_strided(ptr, n, static_cast<int>(blockIdx.x), huge_blocks, op, scratch, list);
    else
        walk_rows<GROUP>(ptr, n, op, nullptr, huge_blocks, huge_blocks > 0, rows_per_wave);
    tango_block_max_update(op.amax, absmax_alpha);
}

// Backward over the in-edges of each destination (steps 4' and 3''): alpha is recomputed from the row statistics,
// P[v][h] = sum dalpha*alpha (fp64), dE = alpha*(dalpha - P), dD[v][h] = sum dE*lrelu'(t).
template <int H>
struct attn_bwd_dst_op {
    const int32_t *src;
    const int8_t *Sq, *Dq;
    float sS, sD, slope;
    const float *row_lse, *dalpha;
    void *rec;
    float *dD;
    template <class Team>
    __device__ void run(int row, int b, int t, Team tm)
    {
        float td[H], lse[H];
        double p[H], acc[H];
        int dq[H];
        tango_load_heads<H>(Dq, row, dq);
#pragma unroll
        for (int h = 0; h < H; ++h) {
            td[h] = sD * static_cast<float>(dq[h]);
            lse[h] = row_lse[static_cast<int64_t>(row) * H + h];
            p[h] = 0.0;
            acc[h] = 0.0;
        }
        for (int e = b + tm.rank; e < t; e += tm.size()) {
            int sq[H];
            tango_load_heads<H>(Sq, src[e], sq);
            float d[H];
            load_h<H>(dalpha + static_cast<int64_t>(e) * H, d);
#pragma unroll
            for (int h = 0; h < H; ++h) {
                bool pos;
                const float ev = tango_attn_score(sS * static_cast<float>(sq[h]), td[h], slope, pos);
                const float al = tango_attn_alpha(ev, lse[h]);
                p[h] += static_cast<double>(d[h]) * static_cast<double>(al);
            }
        }
#pragma unroll
        for (int h = 0; h < H; ++h) p[h] = tm.sum(p[h]);
        for (int e = b + tm.rank; e < t; e += tm.size()) {
            int sq[H];
            tango_load_heads<H>(Sq, src[e], sq);
            float d[H];
            load_h<H>(dalpha + static_cast<int64_t>(e) * H, d);
#pragma unroll
            for (int h = 0; h < H; ++h) {
                bool pos;
                const float ev = tango_attn_score(sS * static_cast<float>(sq[h]), td[h], slope, pos);
                const float al = tango_attn_alpha(ev, lse[h]);
                const float dE = static_cast<float>(static_cast<double>(al) * (static_cast<double>(d[h]) - p[h]));
                acc[h] += static_cast<double>(dE * (pos ? 1.0f : slope));
            }
        }
#pragma unroll
        for (int h = 0; h < H; ++h) {
            const double sacc = tm.sum(acc[h]);
            if (tm.rank == 0) {
                tango_attn_rec rc;
                rc.P = p[h];
                rc.row_lse = lse[h];
                rc.dq = dq[h];
                static_cast<tango_attn_rec *>(rec)[static_cast<int64_t>(row) * tango_rec_heads(H) + h] = rc;
                dD[static_cast<int64_t>(row) * H + h] = static_cast<float>(sacc);
            }
        }
    }
};

template <int H, int GROUP>
__global__ __launch_bounds__(256) void k_attn_bwd_dst(int n, const int32_t *ptr, attn_bwd_dst_op<H> op, const float *sS,
                                                      const float *sD, int *huge)
{
    op.sS = *sS;
    op.sD = *sD;
    walk_rows<GROUP>(ptr, n, op, huge);
}

template <int H>
__global__ __launch_bounds__(TEAM_BLOCK_THREADS) void k_attn_bwd_dst_huge(const int32_t *ptr, attn_bwd_dst_op<H> op,
                                                                          const float *sS, const float *sD,
                                                                          const int *huge)
{
    __shared__ double scratch[2 * TEAM_BLOCK_THREADS / 64];
    op.sS = *sS;
    op.sD = *sD;
    walk_huge_rows(ptr, huge, op, scratch);
}

}  // namespace

int tango_attn_bwd_dst_async(const tango_graph *g, int heads, const int8_t *Sq, const float *sS, const int8_t *Dq,
                             const float *sD, float slope, const float *row_lse,
                             const float *dalpha, void *rec, float *dD, int *huge, hipStream_t st)
{
    const int n = g->n_nodes;
    const int grp = pick_group(n, g->n_edges);
    const unsigned grid = row_grid(n, grp);
    int rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(huge), 0u, 1, st);
    if (rc != TANGO_OK) return rc;
#define CALL(HH)                                                                                            \
    {                                                                                                       \
        attn_bwd_dst_op<HH> op{g->in_src, Sq, Dq, 0.f, 0.f, slope, row_lse, dalpha, rec, dD};        \
        k_attn_bwd_dst<HH, GROUP><<<grid, 256, 0, st>>>(n, g->in_ptr, op, sS, sD, huge);                    \
        k_attn_bwd_dst_huge<HH><<<HUGE_GRID, TEAM_BLOCK_THREADS, 0, st>>>(g->in_ptr, op, sS, sD, huge);      \
    }
    TANGO_DISPATCH_H(heads, grp, CALL)
#undef CALL
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

int tango_attn_stats_async(const tango_graph *g, int heads, const int8_t *Sq, const float *sS, const int8_t *Dq,
                           const float *sD, float slope, float *row_lse, float *absmax_alpha,
                           int *huge, int8_t *src_codes, bool absmax_zeroed, hipStream_t st)
{
    (void)huge;  // (the list of long rows is only used by the backward walk; here they are found inside the launch)
    const int n = g->n_nodes;
    const int grp = pick_group(n, g->n_edges);
    const int rpw = pick_rows_per_wave(n, grp);
    const unsigned grid = row_grid(n, grp, rpw);
    if (!absmax_zeroed) {
        int rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(absmax_alpha), 0u, 1, st);
        if (rc != TANGO_OK) return rc;
    }
    // no row can be longer than HUGE_ROW unless the graph has that many edges
    const int huge_blocks = g->n_edges > HUGE_ROW ? static_cast<int>(std::min<int64_t>(HUGE_GRID, n)) : 0;
#define CALL(HH)                                                                                             \
    {                                                                                                        \
        attn_stats_op<HH> op{g->in_src, Sq, Dq, 0.f, 0.f, slope, row_lse, 0.f, src_codes};                   \
        k_attn_stats<HH, GROUP><<<grid + huge_blocks, 256, 0, st>>>(n, g->in_ptr, op, sS, sD, absmax_alpha, huge_blocks, rpw); \
    }
    TANGO_DISPATCH_H(heads, grp, CALL)
#undef CALL
    TANGO_LAUNCH_CHECK();
    return TANGO_OK;
}

extern "C" {

size_t tango_gat_attention_workspace_bytes(int64_t, int64_t n_edges, int) { return 256 + huge_list_bytes(n_edges); }

int tango_gat_attention_fwd(const tango_graph *g, int heads, int dim, const int8_t *S_q, const float *s_S,
                            const int8_t *D_q, const float *s_D, float slope, const int8_t *X_q, const float *s_X,
                            int rounding, uint64_t seed, uint64_t stream_id_alpha, float *row_lse, int8_t *alpha_q,
                            float *s_alpha, float *absmax_alpha, float *alpha_dump, float *out, float *absmax_out,
                            void *ws, size_t ws_bytes, void *stream)
{
    return tango_gat_attention_fwd_act(g, heads, dim, S_q, s_S, D_q, s_D, slope, X_q, s_X, rounding, seed, stream_id_alpha,
                                       row_lse, alpha_q, s_alpha, absmax_alpha, alpha_dump, out, absmax_out, 0, nullptr, nullptr,
                                       ws, ws_bytes, stream);
}

}  // extern "C"

// tango_gat_attention_fwd with an optional ReLU on the aggregate (relu_out != 0: out = max(0, .), absmax_out of that).
// relu_bits (optional, 8-byte aligned, n*heads*dim/8 bytes, only where tango_spmm_relu_bits_supported): bit i of the flat
// output is set where out[i] > 0.
// src_codes (optional, 8-byte aligned, n_edges*heads bytes): receives S_q[src(e)] of every in-edge e, in edge order, from the
// statistics pass; the aggregation pass (and the backward pass, if handed the same buffer) then reads these in a
// stream instead of gathering from S_q once more per edge.
int tango_gat_attention_fwd_act(const tango_graph *g, int heads, int dim, const int8_t *S_q, const float *s_S,
                                const int8_t *D_q, const float *s_D, float slope, const int8_t *X_q, const float *s_X,
                                int rounding, uint64_t seed, uint64_t stream_id_alpha, float *row_lse, int8_t *alpha_q,
                                float *s_alpha, float *absmax_alpha, float *alpha_dump, float *out, float *absmax_out,
                                int relu_out, void *relu_bits, int8_t *src_codes, void *ws, size_t ws_bytes, void *stream,
                                bool absmax_alpha_zeroed, bool out_prezeroed)
{
    TANGO_REQUIRE(rounding == TANGO_RN || rounding == TANGO_SR, TANGO_ERR_BAD_ENUM);
    TANGO_REQUIRE(g != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(g->n_nodes > 0 && g->n_edges >= 0 && g->n_edges < (int64_t(1) << 31), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(g->in_ptr && (g->n_edges == 0 || g->in_src), TANGO_ERR_NULL);
    TANGO_REQUIRE(heads_supported(heads), TANGO_ERR_UNSUPPORTED);
    int rc = tango_validate_spmm_shape(heads, dim);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(S_q && s_S && D_q && s_D && X_q && s_X && row_lse && s_alpha && absmax_alpha && out, TANGO_ERR_NULL);
    TANGO_REQUIRE(!relu_bits || (relu_out && tango_aligned(relu_bits, 8) &&
                                 tango_spmm_relu_bits_supported(g->n_nodes, heads, dim)),
                  TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(tango_aligned(out, 16) && tango_aligned(X_q, 16) && tango_aligned(src_codes, 8), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(ws && tango_aligned(ws, 256) &&
                      ws_bytes >= tango_gat_attention_workspace_bytes(g->n_nodes, g->n_edges, heads),
                  TANGO_ERR_WORKSPACE);
    TANGO_REQUIRE(tango_aligned(S_q, heads == 3 ? 1 : heads) && tango_aligned(D_q, heads == 3 ? 1 : heads), TANGO_ERR_BAD_SHAPE);
    hipStream_t st = tango_stream(stream);
    int *huge = reinterpret_cast<int *>(static_cast<char *>(ws) + 256);
    if (g->n_edges == 0) {  // no edge: the scale of an empty tensor is 1
        rc = tango_fill_u32_async(reinterpret_cast<uint32_t *>(s_alpha), 0x3f800000u, 1, st);
        if (rc != TANGO_OK) return rc;
    }
    rc = tango_attn_stats_async(g, heads, S_q, s_S, D_q, s_D, slope, row_lse, absmax_alpha, huge, src_codes, absmax_alpha_zeroed,
                                st);
    if (rc != TANGO_OK) return rc;
    return tango_spmm_attention_async(g, TANGO_IN, heads, dim, S_q, s_S, D_q, s_D, slope, row_lse, absmax_alpha, rounding,
                                      seed, stream_id_alpha, alpha_q, s_alpha, alpha_dump, X_q, s_X, out, absmax_out, relu_out,
                                      static_cast<uint16_t *>(relu_bits), src_codes, st, out_prezeroed);
}

extern "C" {

size_t tango_gat_attention_bwd_workspace_bytes(int64_t n_nodes, int64_t n_edges, int heads)
{
    // the per-destination records (P, row_lse); per (node, head) a double dS accumulator and three running sums; then
    // the list of hub rows
    return 256 + tango_gat_attention_bwd_rec_bytes(n_nodes, heads) +
           4 * tango_round_up(static_cast<size_t>(n_nodes) * heads * sizeof(double), 256) + huge_list_bytes(n_edges);
}

size_t tango_gat_attention_bwd_rec_bytes(int64_t n_nodes, int heads)
{
    return tango_round_up(static_cast<size_t>(n_nodes) * tango_rec_heads(heads) * sizeof(tango_attn_rec), 256);
}

size_t tango_gat_attention_bwd_dst_workspace_bytes(int64_t n_nodes, int heads)
{
    return 3 * tango_round_up(static_cast<size_t>(n_nodes) * heads * sizeof(double), 256);
}

size_t tango_gat_attention_bwd_src_workspace_bytes(int64_t n_nodes, int heads)
{
    return tango_round_up(static_cast<size_t>(n_nodes) * heads * sizeof(double), 256);
}

static int attention_bwd_common_checks(const tango_graph *g, int heads, int dim)
{
    TANGO_REQUIRE(g != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(g->n_nodes > 0 && g->n_edges >= 0 && g->n_edges < (int64_t(1) << 31), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(g->in_ptr && g->out_ptr && (g->n_edges == 0 || (g->in_src && g->out_dst && g->out_eid)), TANGO_ERR_NULL);
    TANGO_REQUIRE(heads_supported(heads), TANGO_ERR_UNSUPPORTED);
    return tango_validate_sddmm_dot_shape(heads, dim);
}

int tango_gat_attention_bwd_dst(const tango_graph *g, int heads, int dim, const int8_t *S_q, const float *s_S,
                                const int8_t *D_q, const float *s_D, float slope, const float *row_lse, const int8_t *X_q,
                                const float *s_X, const int8_t *dOut_q, const float *s_dOut, void *rec, float *dD, void *ws,
                                size_t ws_bytes, void *stream)
{
    int rc = attention_bwd_common_checks(g, heads, dim);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(S_q && s_S && D_q && s_D && row_lse && X_q && s_X && dOut_q && s_dOut && rec && dD, TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(S_q, heads == 3 ? 1 : heads) && tango_aligned(D_q, heads == 3 ? 1 : heads), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(tango_aligned(X_q, 16) && tango_aligned(dOut_q, 16) && tango_aligned(rec, 16), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(ws && tango_aligned(ws, 256) && ws_bytes >= tango_gat_attention_bwd_dst_workspace_bytes(g->n_nodes, heads),
                  TANGO_ERR_WORKSPACE);
    return tango_attn_bwd_dst_fused_async(g, heads, dim, dOut_q, s_dOut, X_q, s_X, S_q, s_S, D_q, s_D, slope, row_lse,
                                          static_cast<double *>(ws), rec, dD, nullptr, nullptr, false,
                                          tango_stream(stream));
}

int tango_gat_attention_bwd_src(const tango_graph *g, int heads, int dim, const int8_t *S_q, const float *s_S,
                                const int8_t *D_q, const float *s_D, float slope, const float *row_lse, const float *s_alpha,
                                const float *absmax_alpha, int rounding, uint64_t seed, uint64_t stream_id_alpha,
                                const int8_t *X_q, const float *s_X, const int8_t *dOut_q, const float *s_dOut,
                                const void *rec, float *dX_agg, float *absmax_dX, float *dS, void *ws, size_t ws_bytes,
                                void *stream)
{
    TANGO_REQUIRE(rounding == TANGO_RN || rounding == TANGO_SR, TANGO_ERR_BAD_ENUM);
    int rc = attention_bwd_common_checks(g, heads, dim);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(S_q && s_S && D_q && s_D && row_lse && s_alpha && absmax_alpha && X_q && s_X && dOut_q && s_dOut && rec &&
                      dX_agg && dS,
                  TANGO_ERR_NULL);
    TANGO_REQUIRE(tango_aligned(X_q, 16) && tango_aligned(dOut_q, 16) && tango_aligned(rec, 16) && tango_aligned(dX_agg, 16),
                  TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(ws && tango_aligned(ws, 256) && ws_bytes >= tango_gat_attention_bwd_src_workspace_bytes(g->n_nodes, heads),
                  TANGO_ERR_WORKSPACE);
    return tango_spmm_attention_rev_ds_async(g, heads, dim, S_q, s_S, D_q, s_D, slope, row_lse, absmax_alpha, rounding, seed,
                                             stream_id_alpha, s_alpha, dOut_q, s_dOut, X_q, s_X,
                                             rec, static_cast<double *>(ws), dX_agg,
                                             absmax_dX, dS, false, tango_stream(stream));
}

int tango_gat_attention_bwd(const tango_graph *g, int heads, int dim, const int8_t *S_q, const float *s_S,
                            const int8_t *D_q, const float *s_D, float slope, const float *row_lse, const int8_t *alpha_q,
                            const float *s_alpha, const float *absmax_alpha, int rounding, uint64_t seed,
                            uint64_t stream_id_alpha, const int8_t *X_q, const float *s_X, const int8_t *dOut_q,
                            const float *s_dOut, float *dX_agg, float *absmax_dX, float *dalpha, float *dS, float *dD,
                            void *ws, size_t ws_bytes, void *stream)
{
    return tango_gat_attention_bwd_cached(g, heads, dim, S_q, s_S, D_q, s_D, slope, row_lse, alpha_q, s_alpha, absmax_alpha,
                                          rounding, seed, stream_id_alpha, X_q, s_X, dOut_q, s_dOut, dX_agg, absmax_dX, dalpha,
                                          dS, dD, nullptr, ws, ws_bytes, stream);
}

}  // extern "C"

// What tango_gat_attention_bwd_cached clears before its first kernel when it keeps no edge tensor: the accumulator of
// dS and the three running sums per (node, head), which lie side by side in its workspace.
void tango_gat_attention_bwd_zero_regions(const tango_graph *g, int heads, void *ws, tango_zero_regions &z)
{
    const int64_t nh = static_cast<int64_t>(g->n_nodes) * heads;
    const size_t nh_bytes = tango_round_up(static_cast<size_t>(nh) * sizeof(double), 256);
    const size_t rec_bytes = tango_gat_attention_bwd_rec_bytes(g->n_nodes, heads);
    tango_zero_regions_add(z, static_cast<char *>(ws) + 256 + rec_bytes, 2 * nh);             // dS_acc
    tango_zero_regions_add(z, static_cast<char *>(ws) + 256 + rec_bytes + nh_bytes, 6 * nh);  // stats
}

// tango_gat_attention_bwd with the edge-ordered source codes the forward pass left (src_codes, may be NULL): the walk over
// the in-edges then reads them in a stream instead of gathering from S_q.
int tango_gat_attention_bwd_cached(const tango_graph *g, int heads, int dim, const int8_t *S_q, const float *s_S,
                                   const int8_t *D_q, const float *s_D, float slope, const float *row_lse,
                                   const int8_t *alpha_q, const float *s_alpha, const float *absmax_alpha, int rounding,
                                   uint64_t seed, uint64_t stream_id_alpha, const int8_t *X_q, const float *s_X,
                                   const int8_t *dOut_q, const float *s_dOut, float *dX_agg, float *absmax_dX, float *dalpha,
                                   float *dS, float *dD, const int8_t *src_codes, void *ws, size_t ws_bytes, void *stream,
                                   bool prezeroed, bool out_prezeroed)
{
    TANGO_REQUIRE(rounding == TANGO_RN || rounding == TANGO_SR, TANGO_ERR_BAD_ENUM);
    TANGO_REQUIRE(g != nullptr, TANGO_ERR_NULL);
    TANGO_REQUIRE(g->n_nodes > 0 && g->n_edges >= 0 && g->n_edges < (int64_t(1) << 31), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(g->in_ptr && g->out_ptr && (g->n_edges == 0 || (g->in_src && g->out_dst && g->out_eid)), TANGO_ERR_NULL);
    TANGO_REQUIRE(heads_supported(heads), TANGO_ERR_UNSUPPORTED);
    int rc = tango_validate_sddmm_dot_shape(heads, dim);
    if (rc != TANGO_OK) return rc;
    TANGO_REQUIRE(S_q && s_S && D_q && s_D && row_lse && s_alpha && absmax_alpha && X_q && s_X && dOut_q && s_dOut &&
                      dX_agg,
                  TANGO_ERR_NULL);
    const bool edge_part = dalpha || dS || dD;
    TANGO_REQUIRE(!edge_part || (dS && dD), TANGO_ERR_NULL);
    TANGO_REQUIRE(!(alpha_q && edge_part && g->n_edges > 0 && !dalpha), TANGO_ERR_NULL);  // the cached-codes path keeps dalpha
    TANGO_REQUIRE(tango_aligned(dX_agg, 16) && tango_aligned(X_q, 16) && tango_aligned(dOut_q, 16) &&
                      tango_aligned(dalpha, 16) && tango_aligned(src_codes, 8),
                  TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(tango_aligned(S_q, heads == 3 ? 1 : heads) && tango_aligned(D_q, heads == 3 ? 1 : heads), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(ws && tango_aligned(ws, 256) &&
                      ws_bytes >= tango_gat_attention_bwd_workspace_bytes(g->n_nodes, g->n_edges, heads),
                  TANGO_ERR_WORKSPACE);
    hipStream_t st = tango_stream(stream);
    const size_t nh_bytes = tango_round_up(static_cast<size_t>(g->n_nodes) * heads * sizeof(double), 256);
    const size_t rec_bytes = tango_gat_attention_bwd_rec_bytes(g->n_nodes, heads);
    void *rec = static_cast<char *>(ws) + 256;
    double *dS_acc = reinterpret_cast<double *>(static_cast<char *>(ws) + 256 + rec_bytes);
    double *stats = reinterpret_cast<double *>(static_cast<char *>(ws) + 256 + rec_bytes + nh_bytes);
    int *huge = reinterpret_cast<int *>(static_cast<char *>(ws) + 256 + rec_bytes + 4 * nh_bytes);
    if (edge_part && !alpha_q && !dalpha) {
        // no edge tensor at all: 5'', 4', 3'' in one walk over the in-edges, then 5' and 3' in one walk over the out-edges
        rc = tango_attn_bwd_dst_fused_async(g, heads, dim, dOut_q, s_dOut, X_q, s_X, S_q, s_S, D_q, s_D, slope, row_lse, stats,
                                            rec, dD, src_codes, dS_acc, prezeroed, st);
        if (rc != TANGO_OK) return rc;
        return tango_spmm_attention_rev_ds_async(g, heads, dim, S_q, s_S, D_q, s_D, slope, row_lse, absmax_alpha, rounding, seed,
                                                 stream_id_alpha, s_alpha, dOut_q, s_dOut, X_q, s_X, rec, dS_acc, dX_agg,
                                                 absmax_dX, dS, true, st, out_prezeroed);
    }
    if (edge_part && !alpha_q) {
        // 5'' over in-edges (dalpha, the only fp32 edge tensor of the backward pass), 4' and 3'' over in-edges, then
        // 5' and 3' together in one walk over the out-edges: both need the rows dOut_q[v] of every out-edge (u -> v)
        rc = tango_sddmm_dot_async(g, heads, dim, dOut_q, s_dOut, X_q, s_X, dalpha, st);
        if (rc != TANGO_OK) return rc;
        rc = tango_attn_bwd_dst_async(g, heads, S_q, s_S, D_q, s_D, slope, row_lse, dalpha, rec, dD, huge, st);
        if (rc != TANGO_OK) return rc;
        return tango_spmm_attention_rev_ds_async(g, heads, dim, S_q, s_S, D_q, s_D, slope, row_lse, absmax_alpha, rounding, seed,
                                                 stream_id_alpha, s_alpha, dOut_q, s_dOut, X_q, s_X, rec, dS_acc, dX_agg,
                                                 absmax_dX, dS, false, st);
    }
    // 5': SPMM on the reversed graph.  With a cached alpha_q its codes are read through the edge-id map (a random
    // 4-byte access per edge); without, the identical codes are recomputed from the cache-resident S_q, D_q, row_lse.
    if (alpha_q)
        rc = tango_spmm_async(g, TANGO_OUT, heads, dim, alpha_q, s_alpha, dOut_q, s_dOut, dX_agg, absmax_dX, st);
    else
        rc = tango_spmm_attention_async(g, TANGO_OUT, heads, dim, S_q, s_S, D_q, s_D, slope, row_lse, absmax_alpha, rounding,
                                        seed, stream_id_alpha, nullptr, const_cast<float *>(s_alpha), nullptr, dOut_q,
                                        s_dOut, dX_agg, absmax_dX, 0, nullptr, nullptr, st);
    if (rc != TANGO_OK || !edge_part) return rc;
    // 5'': dalpha, the only fp32 edge tensor of the backward pass
    rc = tango_sddmm_dot_async(g, heads, dim, dOut_q, s_dOut, X_q, s_X, dalpha, st);
    if (rc != TANGO_OK) return rc;
    // 4' and 3'' over in-edges, then 3' over out-edges
    rc = tango_attn_bwd_dst_async(g, heads, S_q, s_S, D_q, s_D, slope, row_lse, dalpha, rec, dD, huge, st);
    if (rc != TANGO_OK) return rc;
    return tango_attn_bwd_src_async(g, heads, dim, dOut_q, s_dOut, X_q, s_X, S_q, s_S, D_q, s_D, slope, rec, dS_acc, dS, st);
}


