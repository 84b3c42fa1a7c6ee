// Whole-layer entry points: the primitives chained on one stream with every
// quantized tensor produced once and reused (Sec. 3.3 "Inter-primitive
// optimization").  Host-side sequencing only; all arithmetic is in the kernels
// of the primitives.
#include "internal.hip.h"

namespace {

// random-stream ids of the tensors of one layer (layer l uses 16*l + id)
enum { SID_H = 1, SID_W = 2, SID_HP = 3, SID_S = 4, SID_D = 5, SID_ALPHA = 6, SID_G = 7, SID_DHP = 8 };

// layout of the layer workspace: 256 bytes of scalars, 256 bytes of partial maxima (small tensors' abs-max without
// atomics), the column-sum accumulators of step 2' (outside the shared
// part, so that the backward pass can clear them in its first launch), then the largest sub-call workspace
// (S and D are updated by one kernel at the same time: kept in different 128-byte lines)
enum { SC_ABSMAX_S = 0, SC_ABSMAX_D = 32, SC_ABSMAX_ALPHA = 16, SC_ABSMAX_G = 48 };

constexpr size_t HDR = 512;                 // scalars + partial maxima
constexpr int64_t SMALL_OUT_WORDS = 65536;  // outputs up to this size are cleared whole by the first launch of a chain

size_t max3(size_t a, size_t b, size_t c) { return a > b ? (a > c ? a : c) : (b > c ? b : c); }

#define TANGO_TRY(expr)             \
    do {                            \
        int rc_ = (expr);           \
        if (rc_ != TANGO_OK) return rc_; \
    } while (0)

// whether the ReLU between layers is carried as sign bits (forward SPMM epilogue writes them, backward quantize reads them)
bool gat_uses_relu_bits(const tango_gat_layer *L)
{
    return L->fused && L->relu_out && L->relu_bits && tango_aligned(L->relu_bits, 8) &&
           tango_spmm_relu_bits_supported(L->g->n_nodes, L->heads, L->dim);
}

}  // namespace

extern "C" {

size_t tango_gat_layer_workspace_bytes(int64_t n_nodes, int64_t n_edges, int k_in, int heads, int dim)
{
    const int64_t F = static_cast<int64_t>(heads) * dim;
    const size_t a = tango_qgemm_workspace_bytes(n_nodes, F, k_in);
    const size_t b = tango_qgemm_bwd_workspace_bytes(n_nodes, F, k_in);
    const size_t c = tango_head_proj_bwd_workspace_bytes(n_nodes, heads, dim);
    const size_t d = tango_gat_attention_bwd_workspace_bytes(n_nodes, n_edges, heads);
    const size_t e = tango_gat_attention_workspace_bytes(n_nodes, n_edges, heads);
    return HDR + c + max3(a, b, max3(d, e, 0));
}

int tango_gat_layer_fwd(const tango_gat_layer *L, void *stream)
{
    TANGO_REQUIRE(L && L->g, TANGO_ERR_NULL);
    TANGO_REQUIRE(L->k_in >= 1 && L->heads >= 1 && L->dim >= 1, TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(L->H && L->W && L->a_src && L->a_dst && L->H_q && L->s_H && L->W_q && L->s_W && L->Hp && L->absmax_Hp &&
                      L->Hp_q && L->s_Hp && L->S && L->D && L->S_q && L->s_S && L->D_q && L->s_D && L->s_alpha && L->out,
                  TANGO_ERR_NULL);
    TANGO_REQUIRE(L->fused ? (L->row_lse && L->absmax_alpha) : (L->E && L->alpha && L->alpha_q), TANGO_ERR_NULL);
    const int64_t n = L->g->n_nodes, nnz = L->g->n_edges;
    const int64_t F = static_cast<int64_t>(L->heads) * L->dim;
    TANGO_REQUIRE(L->ws && tango_aligned(L->ws, 256) &&
                      L->ws_bytes >= tango_gat_layer_workspace_bytes(n, nnz, L->k_in, L->heads, L->dim),
                  TANGO_ERR_WORKSPACE);
    float *sc = static_cast<float *>(L->ws);
    const size_t hpb = tango_head_proj_bwd_workspace_bytes(n, L->heads, L->dim);
    void *sub = static_cast<char *>(L->ws) + HDR + hpb;
    const size_t sub_bytes = L->ws_bytes - HDR - hpb;
    const uint64_t sid = 16 * L->layer_id;
    const bool proj_fused = tango_head_proj_quantize_supported(L->heads, L->dim) && tango_aligned(L->Hp, 16) &&
                            tango_aligned(L->Hp_q, 8) && tango_aligned(L->a_src, 16) && tango_aligned(L->a_dst, 16);

    // step 1: H' = H.W, quantize-on-load, cached H_q / W_q, fused abs-max of H'.  Its first launch also clears the
    // abs-max words that steps 2 and 4 accumulate into (each clear of its own would be one more launch in the chain).
    tango_zero_regions zr{};
    if (proj_fused) {
        tango_zero_regions_add(zr, sc + SC_ABSMAX_S, 1);
        tango_zero_regions_add(zr, sc + SC_ABSMAX_D, 1);
    }
    if (L->fused) tango_zero_regions_add(zr, L->absmax_alpha, 1);
    // small graphs: the same launch clears the whole output (a few thousand words), which spares the aggregation its own
    // launch for clearing the rows it adds to
    const bool out_prezero = L->fused && n * F <= SMALL_OUT_WORDS;
    if (out_prezero) {
        tango_zero_regions_add(zr, L->out, n * F);
        tango_zero_regions_add(zr, L->absmax_out, 1);
        if (gat_uses_relu_bits(L)) tango_zero_regions_add(zr, L->relu_bits, n * F / 32);
    }
    TANGO_TRY(tango_qgemm_known_absmax(n, F, L->k_in, L->H, L->absmax_H, L->W, L->rounding, L->seed, sid + SID_H, sid + SID_W,
                                       L->H_q, L->s_H, L->W_q, L->s_W, L->Hp, L->absmax_Hp, sub, sub_bytes, stream, &zr));
    // step 2: S, D in fp32, with their abs-max
    // and the sequential quantization of the tensors the sparse primitives will access randomly (Sec. 3.3): H' in the
    // same pass over H' where the shape allows
    if (proj_fused) {
        TANGO_TRY(tango_head_proj_quantize_async(n, L->heads, L->dim, L->Hp, L->a_src, L->a_dst, L->S, L->D, sc + SC_ABSMAX_S,
                                                 sc + SC_ABSMAX_D, L->absmax_Hp, L->rounding, L->seed, sid + SID_HP, L->Hp_q,
                                                 L->s_Hp, tango_stream(stream), true));
    } else {
        TANGO_TRY(tango_head_proj(n, L->heads, L->dim, L->Hp, L->a_src, L->a_dst, L->S, L->D, sc + SC_ABSMAX_S,
                                  sc + SC_ABSMAX_D, stream));
        TANGO_TRY(tango_quantize(L->Hp, static_cast<size_t>(n * F), L->rounding, L->seed, sid + SID_HP, L->absmax_Hp,
                                 L->Hp_q, L->s_Hp, nullptr, 0, stream));
    }
    TANGO_TRY(tango_quantize_pair_with_absmax_async(L->S, static_cast<size_t>(n * L->heads), sid + SID_S, sc + SC_ABSMAX_S, L->S_q,
                                                    L->s_S, L->D, static_cast<size_t>(n * L->heads), sid + SID_D,
                                                    sc + SC_ABSMAX_D, L->D_q, L->s_D, L->rounding, L->seed, tango_stream(stream)));
    if (L->fused) {
        // steps 3-5 fused: E and alpha never reach memory in fp32
        return tango_gat_attention_fwd_act(L->g, L->heads, L->dim, L->S_q, L->s_S, L->D_q, L->s_D, L->slope, L->Hp_q, L->s_Hp,
                                           L->rounding, L->seed, sid + SID_ALPHA, L->row_lse, L->alpha_q, L->s_alpha,
                                           L->absmax_alpha, L->alpha, L->out, L->absmax_out, L->relu_out,
                                           gat_uses_relu_bits(L) ? L->relu_bits : nullptr, L->src_codes, sub, sub_bytes,
                                           stream, true, out_prezero);
    }
    // step 3: SDDMM-add with on-the-fly dequantization + LeakyReLU
    TANGO_TRY(tango_qsddmm(L->g, TANGO_SDDMM_ADD_LEAKYRELU, L->heads, 1, L->S_q, L->s_S, L->D_q, L->s_D, L->slope, L->E,
                           stream));
    // step 4: edge softmax in fp32
    TANGO_TRY(tango_edge_softmax(L->g, L->heads, L->E, L->alpha, sc + SC_ABSMAX_ALPHA, stream));
    TANGO_TRY(tango_quantize(L->alpha, static_cast<size_t>(nnz * L->heads), L->rounding, L->seed, sid + SID_ALPHA,
                             sc + SC_ABSMAX_ALPHA, L->alpha_q, L->s_alpha, nullptr, 0, stream));
    // step 5: quantized SPMM
    TANGO_TRY(tango_qspmm(L->g, TANGO_IN, L->heads, L->dim, L->alpha_q, L->s_alpha, L->Hp_q, L->s_Hp, L->out,
                          L->absmax_out, stream));
    if (L->relu_out) TANGO_TRY(tango_relu(L->out, static_cast<size_t>(n * F), L->out, L->absmax_out, stream));
    return TANGO_OK;
}

int tango_gat_layer_bwd(const tango_gat_layer *L, void *stream)
{
    TANGO_REQUIRE(L && L->g, TANGO_ERR_NULL);
    TANGO_REQUIRE(L->grad_out && L->g_q && L->s_g && L->dHp && L->absmax_dHp && L->dS && L->dD && L->dHp_q &&
                      L->s_dHp && L->dW && L->da_src && L->da_dst,
                  TANGO_ERR_NULL);
    TANGO_REQUIRE(L->dalpha || (L->fused && !L->alpha_q) || L->g->n_edges == 0, TANGO_ERR_NULL);
    TANGO_REQUIRE(L->a_src && L->a_dst && L->H_q && L->s_H && L->W_q && L->s_W && L->Hp_q && L->s_Hp && L->S_q && L->s_S &&
                      L->D_q && L->s_D && L->s_alpha,
                  TANGO_ERR_NULL);
    TANGO_REQUIRE(L->fused ? (L->row_lse && L->absmax_alpha) : (L->alpha && L->alpha_q), TANGO_ERR_NULL);
    const int64_t n = L->g->n_nodes, nnz = L->g->n_edges;
    const int64_t F = static_cast<int64_t>(L->heads) * L->dim;
    TANGO_REQUIRE(L->ws && tango_aligned(L->ws, 256) &&
                      L->ws_bytes >= tango_gat_layer_workspace_bytes(n, nnz, L->k_in, L->heads, L->dim),
                  TANGO_ERR_WORKSPACE);
    // (what step 2' needs of its operands, checked before anything is enqueued)
    TANGO_REQUIRE(F <= 1024 && L->dim % 4 == 0 && tango_aligned(L->dHp, 16) && tango_aligned(L->Hp_q, 4) &&
                      tango_aligned(L->a_src, 16) && tango_aligned(L->a_dst, 16),
                  TANGO_ERR_BAD_SHAPE);
    float *sc = static_cast<float *>(L->ws);
    float *partials = sc + 64;  // 64 floats
    void *hp_ws = static_cast<char *>(L->ws) + HDR;
    const size_t hpb = tango_head_proj_bwd_workspace_bytes(n, L->heads, L->dim);
    void *sub = static_cast<char *>(L->ws) + HDR + hpb;
    const size_t sub_bytes = L->ws_bytes - HDR - hpb;
    const uint64_t sid = 16 * L->layer_id;
    hipStream_t st = tango_stream(stream);

    // Everything the backward chain accumulates into is cleared by ONE launch at its head: the accumulator and abs-max
    // of step 2', the abs-max of the upstream gradient (when it has to be found here) and, when the attention part
    // keeps no edge tensor, its per-node sums.
    const bool att_prezero = L->fused && !L->alpha_q && !L->dalpha;
    const bool find_absmax_g = !L->absmax_grad_out && !L->relu_out;
    tango_zero_regions zr{};
    tango_head_proj_bwd_zero_regions(L->heads, L->dim, hp_ws, L->absmax_dHp, zr);
    if (att_prezero) tango_gat_attention_bwd_zero_regions(L->g, L->heads, sub, zr);
    const bool dHp_prezero = att_prezero && n * F <= SMALL_OUT_WORDS;  // (as in the forward pass, for the reverse aggregation)
    if (dHp_prezero) tango_zero_regions_add(zr, L->dHp, n * F);
    // a small upstream gradient whose abs-max has to be found here: the clearing launch also leaves per-workgroup maxima
    // of |grad_out|, which the quantizer reduces - one launch less than clear, abs-max, quantize
    const bool g_partials = find_absmax_g && n * F <= 16 * SMALL_OUT_WORDS && tango_aligned(L->grad_out, 16) && tango_aligned(L->g_q, 8);
    int g_count = 1;
    if (g_partials) {
        TANGO_TRY(tango_absmax_partials_async(L->grad_out, static_cast<size_t>(n * F), partials, &g_count, zr, st));
    } else {
        if (find_absmax_g) tango_zero_regions_add(zr, sc + SC_ABSMAX_G, 1);
        TANGO_TRY(tango_zero_regions_async(zr, st));
    }

    // the upstream gradient is quantized once and shared by steps 5' and 5''
    if (L->absmax_grad_out) {
        // the layer above left max|grad_out| (and, with relu_out, wrote grad_out with this layer's ReLU' applied)
        TANGO_TRY(tango_quantize(L->grad_out, static_cast<size_t>(n * F), L->rounding, L->seed, sid + SID_G, L->absmax_grad_out,
                                 L->g_q, L->s_g, sub, sub_bytes, stream));
    } else if (L->relu_out) {
        // the gradient arrives behind the layer's ReLU: ReLU' (out > 0) is applied while it is quantized
        TANGO_REQUIRE(L->out && tango_aligned(L->grad_out, 16) && tango_aligned(L->out, 16) && tango_aligned(L->g_q, 8),
                      TANGO_ERR_BAD_SHAPE);
        if (gat_uses_relu_bits(L))
            TANGO_TRY(tango_quantize_bitmasked_async(L->grad_out, static_cast<const uint8_t *>(L->relu_bits),
                                                     static_cast<size_t>(n * F), L->rounding, L->seed, sid + SID_G, L->g_q,
                                                     L->s_g, static_cast<float *>(L->ws) + SC_ABSMAX_G, tango_stream(stream)));
        else
            TANGO_TRY(tango_quantize_masked_async(L->grad_out, L->out, static_cast<size_t>(n * F), L->rounding, L->seed,
                                                  sid + SID_G, L->g_q, L->s_g, static_cast<float *>(L->ws) + SC_ABSMAX_G,
                                                  tango_stream(stream)));
    } else if (g_partials) {
        TANGO_TRY(tango_quantize_with_absmax_async(L->grad_out, static_cast<size_t>(n * F), L->rounding, L->seed, sid + SID_G,
                                                   partials, L->g_q, L->s_g, st, g_count));
    } else {
        TANGO_REQUIRE(tango_aligned(L->grad_out, 4), TANGO_ERR_BAD_SHAPE);
        TANGO_TRY(tango_absmax_accumulate_async(L->grad_out, static_cast<size_t>(n * F), sc + SC_ABSMAX_G, st));
        TANGO_TRY(tango_quantize_with_absmax_async(L->grad_out, static_cast<size_t>(n * F), L->rounding, L->seed, sid + SID_G,
                                                   sc + SC_ABSMAX_G, L->g_q, L->s_g, st));
    }
    if (L->fused) {
        // 5', 5'', 4', 3', 3'' from the forward caches; dE is never written
        TANGO_TRY(tango_gat_attention_bwd_cached(L->g, L->heads, L->dim, L->S_q, L->s_S, L->D_q, L->s_D, L->slope, L->row_lse,
                                                 L->alpha_q, L->s_alpha, L->absmax_alpha, L->rounding, L->seed,
                                                 sid + SID_ALPHA, L->Hp_q, L->s_Hp, L->g_q, L->s_g, L->dHp, nullptr, L->dalpha,
                                                 L->dS, L->dD, L->src_codes, sub, sub_bytes, stream, att_prezero, dHp_prezero));
    } else {
    // 5' (SPMM on the reversed graph) and 5'' (SDDMM-dot)
    TANGO_TRY(tango_qspmm_bwd(L->g, L->heads, L->dim, L->alpha_q, L->s_alpha, L->Hp_q, L->s_Hp, L->g_q, L->s_g, L->dHp,
                              nullptr, L->dalpha, stream));
    // 4': softmax backward, in place over dalpha
    TANGO_TRY(tango_edge_softmax_bwd(L->g, L->heads, L->alpha, L->dalpha, L->dalpha, stream));
    // LeakyReLU' and 3', 3'': edge-to-node sums
    TANGO_TRY(tango_qsddmm_bwd(L->g, L->heads, L->S_q, L->s_S, L->D_q, L->s_D, L->slope, L->dalpha, nullptr, L->dS, L->dD,
                               stream));
    }
    // 2' fused with dH' = dH'_agg + dH'_att and its abs-max
    // (its last step, a few hundred additions, rides on the first launch of the GEMM pair where that launch exists)
    tango_colsum_job tail{nullptr, 0, 0, nullptr, nullptr};
    const bool defer_tail = L->dH != nullptr && F <= 2048;
    TANGO_TRY(tango_head_proj_bwd_async(n, L->heads, L->dim, L->dS, L->dD, L->a_src, L->a_dst, L->Hp_q, L->s_Hp, L->dHp, L->dHp,
                                        L->absmax_dHp, L->da_src, L->da_dst, hp_ws, st, true, defer_tail ? &tail : nullptr));
    // 1': both GEMMs from the cached H_q, W_q
    TANGO_REQUIRE((!L->dH_keep_bits && !L->absmax_dH) || L->dH, TANGO_ERR_NULL);
    TANGO_TRY(tango_qgemm_bwd_masked(n, F, L->k_in, L->H_q, L->s_H, L->W_q, L->s_W, L->dHp, L->rounding, L->seed, sid + SID_DHP,
                                     L->absmax_dHp, L->dHp_q, L->s_dHp, L->dH, static_cast<const uint32_t *>(L->dH_keep_bits),
                                     L->absmax_dH, L->dW, sub, sub_bytes, stream, defer_tail ? &tail : nullptr));
    return TANGO_OK;
}

size_t tango_gcn_layer_workspace_bytes(int64_t n_nodes, int64_t, int k_in, int f_out)
{
    const size_t a = tango_qgemm_workspace_bytes(n_nodes, f_out, k_in);
    const size_t b = tango_qgemm_bwd_workspace_bytes(n_nodes, f_out, k_in);
    return 256 + (a > b ? a : b);
}

int tango_gcn_layer_fwd(const tango_gcn_layer *L, void *stream)
{
    TANGO_REQUIRE(L && L->g, TANGO_ERR_NULL);
    TANGO_REQUIRE(L->k_in >= 1 && L->f_out >= 4, TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(L->H && L->W && L->w_q && L->s_w && L->H_q && L->s_H && L->W_q && L->s_W && L->Hp && L->absmax_Hp &&
                      L->Hp_q && L->s_Hp && L->out,
                  TANGO_ERR_NULL);
    const int64_t n = L->g->n_nodes, nnz = L->g->n_edges;
    TANGO_REQUIRE(L->ws && tango_aligned(L->ws, 256) &&
                      L->ws_bytes >= tango_gcn_layer_workspace_bytes(n, nnz, L->k_in, L->f_out),
                  TANGO_ERR_WORKSPACE);
    void *sub = static_cast<char *>(L->ws) + 256;
    const size_t sub_bytes = L->ws_bytes - 256;
    const uint64_t sid = 16 * L->layer_id;
    TANGO_TRY(tango_qgemm(n, L->f_out, L->k_in, L->H, L->W, L->rounding, L->seed, sid + SID_H, sid + SID_W, L->H_q, L->s_H,
                          L->W_q, L->s_W, L->Hp, L->absmax_Hp, sub, sub_bytes, stream));
    TANGO_TRY(tango_quantize(L->Hp, static_cast<size_t>(n) * L->f_out, L->rounding, L->seed, sid + SID_HP, L->absmax_Hp,
                             L->Hp_q, L->s_Hp, nullptr, 0, stream));
    TANGO_TRY(tango_qspmm(L->g, TANGO_IN, 1, L->f_out, L->w_q, L->s_w, L->Hp_q, L->s_Hp, L->out, L->absmax_out, stream));
    return TANGO_OK;
}

int tango_gcn_layer_bwd(const tango_gcn_layer *L, void *stream)
{
    TANGO_REQUIRE(L && L->g, TANGO_ERR_NULL);
    TANGO_REQUIRE(L->grad_out && L->g_q && L->s_g && L->dHp && L->absmax_dHp && L->dHp_q && L->s_dHp && L->dW &&
                      L->w_q && L->s_w && L->H_q && L->s_H && L->W_q && L->s_W,
                  TANGO_ERR_NULL);
    const int64_t n = L->g->n_nodes, nnz = L->g->n_edges;
    TANGO_REQUIRE(L->ws && tango_aligned(L->ws, 256) &&
                      L->ws_bytes >= tango_gcn_layer_workspace_bytes(n, nnz, L->k_in, L->f_out),
                  TANGO_ERR_WORKSPACE);
    void *sub = static_cast<char *>(L->ws) + 256;
    const size_t sub_bytes = L->ws_bytes - 256;
    const uint64_t sid = 16 * L->layer_id;
    TANGO_TRY(tango_quantize(L->grad_out, static_cast<size_t>(n) * L->f_out, L->rounding, L->seed, sid + SID_G, nullptr,
                             L->g_q, L->s_g, sub, sub_bytes, stream));
    if (L->w_q_src_order)
        TANGO_TRY(tango_qspmm(L->g, TANGO_OUT_SRC_ORDER, 1, L->f_out, L->w_q_src_order, L->s_w, L->g_q, L->s_g, L->dHp, L->absmax_dHp,
                              stream));
    else
        TANGO_TRY(tango_qspmm(L->g, TANGO_OUT, 1, L->f_out, L->w_q, L->s_w, L->g_q, L->s_g, L->dHp, L->absmax_dHp, stream));
    TANGO_TRY(tango_qgemm_bwd(n, L->f_out, L->k_in, L->H_q, L->s_H, L->W_q, L->s_W, L->dHp, L->rounding, L->seed,
                              sid + SID_DHP, L->absmax_dHp, L->dHp_q, L->s_dHp, L->dH, L->dW, sub, sub_bytes, stream));
    return TANGO_OK;
}

size_t tango_typed_layer_workspace_bytes(int64_t n_nodes, int64_t n_edges, int n_types, int k_in, int f_out)
{
    return tango_gcn_layer_workspace_bytes(n_nodes, n_edges, k_in, n_types * f_out);
}

int tango_typed_layer_fwd(const tango_typed_layer *L, void *stream)
{
    TANGO_REQUIRE(L && L->g_dst, TANGO_ERR_NULL);
    TANGO_REQUIRE(L->k_in >= 1 && L->f_out >= 4 && L->n_types >= 1, TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(L->H && L->W && L->w_q && L->s_w && L->H_q && L->s_H && L->W_q && L->s_W && L->Hp && L->absmax_Hp &&
                      L->Hp_q && L->s_Hp && L->out,
                  TANGO_ERR_NULL);
    const int64_t n = L->g_dst->n_nodes, nnz = L->g_dst->n_edges;
    const int64_t FT = static_cast<int64_t>(L->n_types) * L->f_out;
    TANGO_REQUIRE(n * L->n_types < (int64_t(1) << 31), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(L->ws && tango_aligned(L->ws, 256) &&
                      L->ws_bytes >= tango_typed_layer_workspace_bytes(n, nnz, L->n_types, L->k_in, L->f_out),
                  TANGO_ERR_WORKSPACE);
    void *sub = static_cast<char *>(L->ws) + 256;
    const size_t sub_bytes = L->ws_bytes - 256;
    const uint64_t sid = 16 * L->layer_id;
    // all type blocks in one GEMM: Z = H.[W_0 | ... | W_{T-1}]
    TANGO_TRY(tango_qgemm(n, FT, L->k_in, L->H, L->W, L->rounding, L->seed, sid + SID_H, sid + SID_W, L->H_q, L->s_H,
                          L->W_q, L->s_W, L->Hp, L->absmax_Hp, sub, sub_bytes, stream));
    TANGO_TRY(tango_quantize(L->Hp, static_cast<size_t>(n * FT), L->rounding, L->seed, sid + SID_HP, L->absmax_Hp, L->Hp_q,
                             L->s_Hp, nullptr, 0, stream));
    // Z_q seen as (n*T) x f_out: in_src of the destination view already names the (source, type) row
    TANGO_TRY(tango_qspmm(L->g_dst, TANGO_IN, 1, L->f_out, L->w_q, L->s_w, L->Hp_q, L->s_Hp, L->out, L->absmax_out,
                          stream));
    return TANGO_OK;
}

int tango_typed_layer_bwd(const tango_typed_layer *L, void *stream)
{
    TANGO_REQUIRE(L && L->g_dst && L->g_src, TANGO_ERR_NULL);
    TANGO_REQUIRE(L->k_in >= 1 && L->f_out >= 4 && L->n_types >= 1, TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(L->grad_out && L->g_q && L->s_g && L->dHp && L->absmax_dHp && L->dHp_q && L->s_dHp && L->dW &&
                      L->w_q && L->s_w && L->H_q && L->s_H && L->W_q && L->s_W,
                  TANGO_ERR_NULL);
    const int64_t n = L->g_dst->n_nodes, nnz = L->g_dst->n_edges;
    const int64_t FT = static_cast<int64_t>(L->n_types) * L->f_out;
    TANGO_REQUIRE(n * L->n_types < (int64_t(1) << 31), TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(L->g_src->n_nodes == n * L->n_types && L->g_src->n_edges == nnz, TANGO_ERR_BAD_SHAPE);
    TANGO_REQUIRE(L->ws && tango_aligned(L->ws, 256) &&
                      L->ws_bytes >= tango_typed_layer_workspace_bytes(n, nnz, L->n_types, L->k_in, L->f_out),
                  TANGO_ERR_WORKSPACE);
    void *sub = static_cast<char *>(L->ws) + 256;
    const size_t sub_bytes = L->ws_bytes - 256;
    const uint64_t sid = 16 * L->layer_id;
    TANGO_TRY(tango_quantize(L->grad_out, static_cast<size_t>(n) * L->f_out, L->rounding, L->seed, sid + SID_G, nullptr,
                             L->g_q, L->s_g, sub, sub_bytes, stream));
    // dZ: one output row per (source, type) pair, i.e. n rows of n_types*f_out
    if (L->w_q_src_order)
        TANGO_TRY(tango_qspmm(L->g_src, TANGO_OUT_SRC_ORDER, 1, L->f_out, L->w_q_src_order, L->s_w, L->g_q, L->s_g, L->dHp,
                              L->absmax_dHp, stream));
    else
        TANGO_TRY(tango_qspmm(L->g_src, TANGO_OUT, 1, L->f_out, L->w_q, L->s_w, L->g_q, L->s_g, L->dHp, L->absmax_dHp, stream));
    TANGO_TRY(tango_qgemm_bwd(n, FT, L->k_in, L->H_q, L->s_H, L->W_q, L->s_W, L->dHp, L->rounding, L->seed, sid + SID_DHP,
                              L->absmax_dHp, L->dHp_q, L->s_dHp, L->dH, L->dW, sub, sub_bytes, stream));
    return TANGO_OK;
}

}  // extern "C"
